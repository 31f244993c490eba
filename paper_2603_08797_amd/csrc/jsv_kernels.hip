// HIP kernels of the allocation search, written for gfx950 (CDNA4, wave64).
//
//   prune_kernel      replicas and cost of every (task, choice) at every level
//                     (Eq. 5-7), then the per-task prune: latency filter, exact
//                     dominance, cap thinning, compaction.
//   mix_kernel        mixture mode: the options of every task (Eq. 2, 6, 7, 9, 10) in place
//                     of prune_kernel.
//   plan_kernel       index strides, packed keys, local keys and the innermost stream,
//                     tile geometry per instance; its last block evens out the tiles,
//                     scans their counts and fixes how they are handed to the blocks.
//   enumerate_kernel  every candidate scored and masked (Eq. 3, 8, 11-13) and
//                     reduced per lane / wave / block to the cheapest feasible one or to
//                     the one with the best objective of Eq. 14; <MODE, BOUNDS>: single
//                     tuples or mixtures, either objective, with or without the bulk
//                     exclusion by bounds.
//   finalize_kernel   grid-level reduction, winner decoded and rescored, sweep summary.
//   eval_kernel       explicit candidates scored one per thread (parity aid).
//
// The enumeration is bound by vector-ALU issue; there is no dense contraction
// anywhere, so no MFMA.  Table entries of the tasks looped inside a lane are
// wave-uniform and are fetched with scalar loads (constant address space) so that
// they feed the vector ALU as scalar operands; the entries that differ per lane are
// gathered from a copy of the instance's tables in LDS.  In the common case a
// candidate costs two vector instructions: a latency compare that narrows the
// execution mask and a minimum on a 32-bit local key (loop_x32_masked, loop_x32).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "jsv_device.h"
#include "jsv_launch.h"

namespace jsv {

#define JSV_CONST __attribute__((address_space(4)))

template <typename T>
__device__ __forceinline__ const T JSV_CONST* as_uniform(const T* p)
{
    return (const T JSV_CONST*)(uintptr_t)p;
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint64_t umin64(uint64_t a, uint64_t b) { return a < b ? a : b; }

// ---- wave64 / block minimum of a u64 key -----------------------------------------------
// Rows of 16 lanes are reduced with DPP (two quad permutes, half-row mirror, row
// mirror), the two 32-lane halves with ds_swizzle, the rest with readlane.
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_min(uint64_t v)
{
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    uint32_t olo = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, 0xF, 0xF, false);
    uint32_t ohi = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, 0xF, 0xF, false);
    return umin64(v, ((uint64_t)ohi << 32) | olo);
}

__device__ __forceinline__ uint64_t wave_min(uint64_t v)
{
    v = dpp_min<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_min<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_min<0x141>(v);   // row_half_mirror
    v = dpp_min<0x140>(v);   // row_mirror: every lane holds its row's minimum
    {                        // lanes i and i^16 of each 32-lane half
        uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
        uint32_t olo = (uint32_t)__builtin_amdgcn_ds_swizzle((int)lo, 0x401F);
        uint32_t ohi = (uint32_t)__builtin_amdgcn_ds_swizzle((int)hi, 0x401F);
        v = umin64(v, ((uint64_t)ohi << 32) | olo);
    }
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    uint64_t a = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi, 0) << 32) |
                 (uint32_t)__builtin_amdgcn_readlane((int)lo, 0);
    uint64_t b = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi, 32) << 32) |
                 (uint32_t)__builtin_amdgcn_readlane((int)lo, 32);
    return umin64(a, b);
}

// Minimum over a 256-thread block; the result is valid in thread 0.
__device__ __forceinline__ uint64_t block_min(uint64_t v, uint64_t* s_red)
{
    v = wave_min(v);
    const uint32_t wave = threadIdx.x >> 6;
    __syncthreads();                       // s_red may still be read from a previous use
    if ((threadIdx.x & 63) == 0) s_red[wave] = v;
    __syncthreads();
    return umin64(umin64(s_red[0], s_red[1]), umin64(s_red[2], s_red[3]));
}

// Objective mode: a lane's best is the pair (objective, key); larger objective wins,
// equal objectives go to the smaller key, i.e. lower cost and then lower index.  "No
// candidate" is (-inf, NO_KEY) and loses against everything.
struct Best { uint64_t key; double obj; };

__device__ __forceinline__ bool better(double ao, uint64_t ak, double bo, uint64_t bk)
{
    return ao > bo || (ao == bo && ak < bk);
}

__device__ __forceinline__ Best pick(const Best& a, const Best& b) { return better(b.obj, b.key, a.obj, a.key) ? b : a; }

template <int CTRL>
__device__ __forceinline__ Best dpp_best(const Best& v)
{
    const uint64_t ob = __builtin_bit_cast(uint64_t, v.obj);
    Best o;
    o.key = ((uint64_t)(uint32_t)__builtin_amdgcn_update_dpp((int)(v.key >> 32), (int)(v.key >> 32), CTRL, 0xF, 0xF, false) << 32) |
            (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)v.key, (int)(uint32_t)v.key, CTRL, 0xF, 0xF, false);
    o.obj = __builtin_bit_cast(double,
            ((uint64_t)(uint32_t)__builtin_amdgcn_update_dpp((int)(ob >> 32), (int)(ob >> 32), CTRL, 0xF, 0xF, false) << 32) |
            (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)ob, (int)(uint32_t)ob, CTRL, 0xF, 0xF, false));
    return pick(v, o);
}

__device__ __forceinline__ uint64_t swz16(uint64_t x)
{
    return ((uint64_t)(uint32_t)__builtin_amdgcn_ds_swizzle((int)(x >> 32), 0x401F) << 32) |
           (uint32_t)__builtin_amdgcn_ds_swizzle((int)(uint32_t)x, 0x401F);
}

__device__ __forceinline__ uint64_t lane_of(uint64_t x, int lane)
{
    return ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(x >> 32), lane) << 32) |
           (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, lane);
}

__device__ __forceinline__ Best wave_best(Best v)
{
    v = dpp_best<0xB1>(v);
    v = dpp_best<0x4E>(v);
    v = dpp_best<0x141>(v);
    v = dpp_best<0x140>(v);
    Best o;
    o.key = swz16(v.key);
    o.obj = __builtin_bit_cast(double, swz16(__builtin_bit_cast(uint64_t, v.obj)));
    v = pick(v, o);
    Best a, b;
    a.key = lane_of(v.key, 0);  a.obj = __builtin_bit_cast(double, lane_of(__builtin_bit_cast(uint64_t, v.obj), 0));
    b.key = lane_of(v.key, 32); b.obj = __builtin_bit_cast(double, lane_of(__builtin_bit_cast(uint64_t, v.obj), 32));
    return pick(a, b);
}

// A double as a 64-bit pattern whose unsigned order is the doubles' order (no NaN here), and back.
__device__ __forceinline__ unsigned long long ordered_bits(double x)
{
    const uint64_t b = __builtin_bit_cast(uint64_t, x);
    return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}
__device__ __forceinline__ double from_ordered_bits(unsigned long long o)
{
    const uint64_t b = (o >> 63) ? (o & 0x7FFFFFFFFFFFFFFFull) : ~o;
    return __builtin_bit_cast(double, b);
}

// Best pair over a 256-thread block; valid in thread 0.
__device__ __forceinline__ Best block_best(Best v, uint64_t* s_key, double* s_obj)
{
    v = wave_best(v);
    const uint32_t wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { s_key[wave] = v.key; s_obj[wave] = v.obj; }
    __syncthreads();
    Best r; r.key = s_key[0]; r.obj = s_obj[0];
    for (int w = 1; w < 4; ++w) { Best o; o.key = s_key[w]; o.obj = s_obj[w]; r = pick(r, o); }
    return r;
}

// ---- prune ------------------------------------------------------------------------------
// One block per (instance, task).  Dynamic LDS: per choice lat, cost, rep (u32),
// acc (f64), two flag bytes.
__global__ void __launch_bounds__(256) prune_kernel(Plan pl)
{
    const uint32_t i = blockIdx.x / pl.t_max;
    const uint32_t t = blockIdx.x % pl.t_max;
    Instance* in = pl.inst + i;
    const Graph* g = pl.graphs + in->problem;
    if (t >= g->T) return;
    const uint32_t C = g->C, V = g->V, PB = g->P * g->B, Bn = g->B, Pn = g->P;
    const uint32_t cap = in->cap;
    const uint32_t tid = threadIdx.x;

    extern __shared__ unsigned char smem[];
    double*   s_acc  = (double*)smem;
    uint32_t* s_lat  = (uint32_t*)(s_acc + C);
    uint32_t* s_cost = s_lat + C;
    uint32_t* s_rep  = s_cost + C;
    uint8_t*  s_a    = (uint8_t*)(s_rep + C);    // alive after the latency filter
    uint8_t*  s_k    = s_a + C;                  // kept
    __shared__ uint32_t s_left, s_flags;
    __shared__ uint64_t s_need;
    if (tid == 0) {
        s_left = 0; s_flags = 0;
        // Eq. 5: demand at the task in micro-requests/s.  Fixed multipliers: R * m_t.  Per-variant
        // factors (Eq. 4): R * m_t at a source, elsewhere the sum over incoming edges of the tail's
        // demand times the factor of the variant the tail is held to, floored per edge; walked in
        // topological order up to this task.
        uint64_t need = (uint64_t)in->demand * g->mult[t];
        if (g->fac != nullptr) {
            uint64_t nd[MAXT];
            const uint32_t last = g->pos_of[t];
            for (uint32_t p = 0; p <= last; ++p) {
                const uint32_t u = g->task_at[p];
                uint64_t r = 0;
                if ((g->src_mask >> p) & 1u) r = (uint64_t)in->demand * g->mult[u];
                else
                    for (uint32_t e = 0; e < g->n_edges; ++e)
                        if (g->e_dst[e] == u) {
                            const uint32_t a = g->e_src[e];
                            const uint32_t hv = in->held[a] == NOT_HELD ? 0u : in->held[a];
                            r += nd[a] * g->fac[(size_t)e * V + hv] / 1000u;     // nd < 2^44, factor < 2^20
                        }
                if (r >= NEED_LIMIT) { s_flags = F_OVERFLOW; r = 0; }
                nd[u] = r;
            }
            need = nd[t];
        }
        s_need = need;
    }
    if (blockIdx.x == 0 && tid == 0) pl.summary->plan_done = 0;     // counted up by the plan kernel
    __syncthreads();

    // Eq. 6, 7: replicas (at least one), cost in partition units
    const uint64_t need = s_need;
    const uint32_t held = in->held[t];
    const uint64_t budget = (uint64_t)in->slo_l;
    const uint64_t through = g->through[t];
    uint32_t* g_rep  = pl.rep  + ((size_t)i * pl.t_max + t) * pl.c_max;
    uint32_t* g_cost = pl.cost + ((size_t)i * pl.t_max + t) * pl.c_max;
    uint32_t my_flags = 0;
    for (uint32_t c = tid; c < C; c += blockDim.x) {
        const uint32_t lat = g->lat[(size_t)t * C + c];
        const uint64_t per = 1000ull * g->thr[(size_t)t * C + c];
        uint64_t rep = need / per + (need % per != 0);
        if (rep < 1) rep = 1;
        uint64_t cost = rep * g->units[(c / Bn) % Pn];
        if (rep > 0xFFFFFFFFull || cost > 0x7FFFFFFFull) { my_flags |= F_OVERFLOW; rep = 1; cost = 1; }
        s_lat[c] = lat; s_cost[c] = (uint32_t)cost; s_rep[c] = (uint32_t)rep;
        s_acc[c] = g->acc[(size_t)t * V + c / PB];
        g_rep[c] = (uint32_t)rep; g_cost[c] = (uint32_t)cost;
        // restrictions of the ablations: variant, partition, static per-task budgets
        bool ok = (g->only_variant[t] == 0xFFFFFFFFu || c / PB == g->only_variant[t]) &&
                  (g->only_part == 0xFFFFFFFFu || (c / Bn) % Pn == g->only_part) &&
                  (held == NOT_HELD || c / PB == held);
        if (ok && g->static_budgets) {
            // q*L <= SLO * lat_ref / lat_path, exactly: both sides are below 2^96
            const unsigned __int128 lhs = (unsigned __int128)((uint64_t)g->q * lat) * g->lat_path[t];
            const unsigned __int128 rhs = (unsigned __int128)budget * g->lat_ref[t];
            ok = lhs <= rhs && cost <= g->unit_budget[t];
        }
        // (a) can this choice meet the latency SLO with every other task at its fastest?
        s_a[c] = ok && (cap == 0 || ((uint64_t)g->q * ((uint64_t)lat + through) <= budget));
    }
    __syncthreads();

    // (b) exact dominance on (latency down, accuracy up, cost down); ties keep the lowest id
    uint32_t kept_here = 0;
    for (uint32_t c = tid; c < C; c += blockDim.x) {
        uint8_t keep = s_a[c];
        if (keep && cap != 0) {
            const uint32_t l = s_lat[c], k = s_cost[c];
            const double a = s_acc[c];
            for (uint32_t o = 0; o < C; ++o) {
                if (o == c || !s_a[o]) continue;
                const uint32_t l2 = s_lat[o], k2 = s_cost[o];
                const double a2 = s_acc[o];
                if (l2 <= l && a2 >= a && k2 <= k) {
                    const bool strict = (l2 < l) || (a2 > a) || (k2 < k);
                    if (strict || o < c) { keep = 0; break; }
                }
            }
        }
        s_k[c] = keep;
        kept_here += keep;
    }
    atomicAdd(&s_left, kept_here);
    __syncthreads();

    // (c) cap thinning: each variant keeps floor(cap/V) choices evenly spaced by latency rank
    if (cap != 0 && s_left > cap) {
        my_flags |= F_TRUNCATED;
        const uint32_t quota = cap / V;
        for (uint32_t c = tid; c < C; c += blockDim.x) {
            uint8_t keep = s_k[c];
            if (keep) {
                const uint32_t v = c / PB, l = s_lat[c];
                uint32_t n = 0, rank = 0;
                for (uint32_t o = v * PB; o < (v + 1) * PB; ++o) {
                    if (!s_k[o]) continue;
                    ++n;
                    if (s_lat[o] < l || (s_lat[o] == l && o < c)) ++rank;
                }
                if (n > quota) {
                    // is rank == floor(j*(n-1)/(quota-1)) for some j < quota ?
                    const uint32_t j = (rank * (quota - 1) + (n - 2)) / (n - 1);
                    keep = (j < quota) && ((j * (n - 1)) / (quota - 1) == rank);
                }
            }
            s_a[c] = keep;
        }
        __syncthreads();
        for (uint32_t c = tid; c < C; c += blockDim.x) s_k[c] = s_a[c];
        __syncthreads();
    }

    // (d) compaction in ascending choice id
    Entry* out = pl.entries + ((size_t)i * pl.t_max + t) * pl.k_max;
    uint32_t total_here = 0;
    for (uint32_t c = tid; c < C; c += blockDim.x) {
        if (!s_k[c]) continue;
        uint32_t pos = 0;
        for (uint32_t o = 0; o < c; ++o) pos += s_k[o];
        Entry e;
        e.lat = s_lat[c]; e.cost = s_cost[c]; e.acc = s_acc[c]; e.key = 0;
        e.rep = s_rep[c]; e.choice = c;
        out[pos] = e;
        ++total_here;
    }
    if (tid == 0) s_left = 0;
    __syncthreads();
    atomicAdd(&s_left, total_here);
    if (my_flags) atomicOr(&s_flags, my_flags);
    __syncthreads();
    if (tid == 0) {
        in->K[t] = s_left;
        uint32_t f = s_flags | (s_left == 0 ? F_EMPTY : 0);
        if (f) atomicOr(&in->flags, f);
        if (f & F_TRUNCATED) atomicOr(&in->trunc_mask, 1u << t);
    }
}

// ---- options of mixture mode ------------------------------------------------------------
// Eq. 9, 10 for two instance types: throughput-weighted mean of the two variants' accuracies.
// Two products, one sum, one quotient, each rounded on its own (no contraction), so that the
// dominance test below sees the same bits as any other plain fp64 evaluation of the formula.
__device__ __forceinline__ double mix_accuracy(uint64_t w1i, double a1, uint64_t w2i, double a2)
{
#pragma clang fp contract(off)
    const double w1 = (double)w1i, w2 = (double)w2i;
    const double p1 = w1 * a1;
    const double p2 = w2 * a2;
    const double num = p1 + p2;
    const double den = w1 + w2;
    return num / den;
}

constexpr uint32_t MIX_MAX_REPLICAS = 65535u;
// Threads per block of mix_kernel: a task's pairs of tuples and their splits are many (10^5 to
// 10^6 options) and the blocks few (levels x tasks), so a block brings as many threads as it can.
constexpr int MIX_THREADS = 1024;

// Per-tuple facts of one task, in LDS.
struct MixTuples {
    const double*   acc;     // accuracy of the tuple's variant
    const uint64_t* h;       // throughput of one replica, micro-requests/s
    const uint32_t* lat;
    const uint32_t* units;
    const uint32_t* cls;     // latency class: number of distinct smaller latencies of the task
    const uint32_t* alone;   // replicas the tuple needs on its own (clamped to 65536)
    const uint8_t*  ok;      // bit0: allowed by the search space and the latency filter
};

// Calls f(cost, latency class, accuracy, id) for every option of the task this thread is
// responsible for: single tuples (id = c) and minimal mixtures of c1 < c2
// (id = C + (c1*C + c2)*65536 + m1).  Options that alone exceed S_avail are skipped.
template <typename F>
__device__ __forceinline__ void mix_visit(const MixTuples& m, uint32_t C, uint64_t need, uint32_t S,
                                          uint32_t tid, uint32_t nthreads, uint32_t& flags, F&& f)
{
    for (uint32_t c = tid; c < C; c += nthreads) {
        if (!(m.ok[c] & 1)) continue;
        const uint64_t rep = need / m.h[c] + (need % m.h[c] != 0);
        const uint64_t r1 = rep < 1 ? 1 : rep;
        if (r1 > S) continue;                               // units >= 1: cost > S_avail
        const uint64_t cost = r1 * m.units[c];
        if (cost > S) continue;
        f((uint32_t)cost, m.cls[c], m.acc[c], (uint64_t)c);
    }
    for (uint32_t k = tid; k < C * C; k += nthreads) {
        const uint32_t c1 = k / C, c2 = k % C;
        if (c2 <= c1 || !(m.ok[c1] & m.ok[c2] & 1)) continue;
        const uint32_t u1 = m.units[c1], u2 = m.units[c2];
        if ((uint64_t)u1 + u2 > S || m.alone[c1] < 2) continue;
        uint32_t m1max = (S - u2) / u1;
        if (m1max > m.alone[c1] - 1) m1max = m.alone[c1] - 1;
        const uint64_t h1 = m.h[c1], h2 = m.h[c2];
        const uint32_t cls = umax(m.cls[c1], m.cls[c2]);
        const double a1 = m.acc[c1], a2 = m.acc[c2];
        for (uint32_t m1 = 1; m1 <= m1max; ++m1) {
            const uint64_t rest = need - (uint64_t)m1 * h1;            // > 0: m1 < alone
            const uint64_t m2max = (S - m1 * u1) / u2;                 // >= 1
            if (__umul64hi(m2max, h2) == 0 && m2max * h2 < rest) continue;   // cannot fit S_avail
            const uint64_t m2 = rest / h2 + (rest % h2 != 0);
            if (m2 > m2max) continue;
            if ((uint64_t)(m1 - 1) * h1 + m2 * h2 >= need) continue;   // one replica of c1 too many
            if (m2 > MIX_MAX_REPLICAS) { flags |= F_OVERFLOW; continue; }
            const uint32_t cost = m1 * u1 + (uint32_t)m2 * u2;
            f(cost, cls, mix_accuracy((uint64_t)m1 * h1, a1, m2 * h2, a2),
              (uint64_t)C + ((uint64_t)c1 * C + c2) * 65536u + m1);
        }
    }
}

// One block per (instance, task): the task's surviving options as Entry records.
// Every option lands in the cell (cost, latency class); a cell keeps its most accurate
// option (lowest id among equals), which dominates the rest of the cell.  A cell survives
// the exact dominance test iff no other non-empty cell with cost <= and class <= has an
// accuracy >=, read off a two-dimensional prefix maximum.  More than cap survivors are
// thinned over a grid of latency bands and accuracy ranks (step (c) below).
__global__ void __launch_bounds__(MIX_THREADS) mix_kernel(Plan pl)
{
    const uint32_t i = blockIdx.x / pl.t_max;
    const uint32_t t = blockIdx.x % pl.t_max;
    const uint32_t tid = threadIdx.x;
    Instance* in = pl.inst + i;
    const Graph* g = pl.graphs + in->problem;
    if (blockIdx.x == 0 && tid == 0) pl.summary->plan_done = 0;     // counted up by the plan kernel
    if (t >= g->T) return;
    const uint32_t C = g->C, V = g->V, PB = g->P * g->B, Bn = g->B, Pn = g->P;
    const uint32_t cap = in->cap, S = g->capacity;

    extern __shared__ unsigned char smem[];
    double*   s_acc   = (double*)smem;
    uint64_t* s_h     = (uint64_t*)(s_acc + C);
    uint32_t* s_lat   = (uint32_t*)(s_h + C);
    uint32_t* s_units = s_lat + C;
    uint32_t* s_cls   = s_units + C;
    uint32_t* s_alone = s_cls + C;
    uint8_t*  s_ok    = (uint8_t*)(s_alone + C);
    __shared__ uint32_t s_flags, s_ncls, s_n, s_kept;
    if (tid == 0) { s_flags = 0; s_ncls = 0; s_n = 0; s_kept = 0; }

    const uint64_t need = (uint64_t)in->demand * g->mult[t];            // micro-requests / s (Eq. 5)
    const uint64_t budget = (uint64_t)in->slo_l, through = g->through[t];
    uint32_t* g_rep  = pl.rep  + ((size_t)i * pl.t_max + t) * pl.c_max;
    uint32_t* g_cost = pl.cost + ((size_t)i * pl.t_max + t) * pl.c_max;
    uint32_t my_flags = 0;
    for (uint32_t c = tid; c < C; c += blockDim.x) {
        const uint32_t lat = g->lat[(size_t)t * C + c];
        const uint64_t per = 1000ull * g->thr[(size_t)t * C + c];
        uint64_t rep = need / per + (need % per != 0);
        if (rep < 1) rep = 1;
        const uint32_t units = g->units[(c / Bn) % Pn];
        uint64_t cost = rep * units;
        if (rep > 0xFFFFFFFFull || cost > 0x7FFFFFFFull) { my_flags |= F_OVERFLOW; rep = 1; cost = 1; }
        g_rep[c] = (uint32_t)rep; g_cost[c] = (uint32_t)cost;
        s_acc[c] = g->acc[(size_t)t * V + c / PB];
        s_h[c] = per; s_lat[c] = lat; s_units[c] = units;
        const bool allowed = (g->only_variant[t] == 0xFFFFFFFFu || c / PB == g->only_variant[t]) &&
                             (g->only_part == 0xFFFFFFFFu || (c / Bn) % Pn == g->only_part);
        // (a) can this tuple meet the latency SLO with every other task at its fastest?  A
        // mixture is as slow as its slower tuple, so it passes iff both tuples do.
        const bool fast = (uint64_t)g->q * ((uint64_t)lat + through) <= budget;
        s_ok[c] = (allowed && fast) ? 1 : 0;
        if (allowed && rep >= 2 && rep - 1 > MIX_MAX_REPLICAS) my_flags |= F_OVERFLOW;
        s_alone[c] = rep > 65536 ? 65536u : (uint32_t)rep;
    }
    __syncthreads();
    // latency classes over all tuples of the task
    for (uint32_t c = tid; c < C; c += blockDim.x) {
        bool first = true;
        for (uint32_t o = 0; o < c; ++o) if (s_lat[o] == s_lat[c]) { first = false; break; }
        if (first) { s_ok[c] |= 2; atomicAdd(&s_ncls, 1u); }
    }
    __syncthreads();
    for (uint32_t c = tid; c < C; c += blockDim.x) {
        uint32_t n = 0;
        for (uint32_t o = 0; o < C; ++o) n += ((s_ok[o] & 2) && s_lat[o] < s_lat[c]) ? 1u : 0u;
        s_cls[c] = n;
    }
    const uint32_t ncls = s_ncls;
    const uint64_t ncell = (uint64_t)(S + 1) * ncls;        // <= pl.mix_cells (host)
    const size_t base = ((size_t)i * pl.t_max + t) * pl.mix_cells;
    uint64_t* c_acc = pl.cell_acc + base;
    uint64_t* c_id  = pl.cell_id + base;
    uint64_t* c_pm  = pl.cell_pm + base;
    uint32_t* c_list = pl.cell_list + base;
    for (uint64_t x = tid; x < ncell; x += blockDim.x) { c_acc[x] = 0; c_id[x] = NO_KEY; }
    __syncthreads();

    MixTuples mt{s_acc, s_h, s_lat, s_units, s_cls, s_alone, s_ok};
    mix_visit(mt, C, need, S, tid, blockDim.x, my_flags,
              [&](uint32_t cost, uint32_t cls, double acc, uint64_t) {
                  atomicMax((unsigned long long*)&c_acc[(uint64_t)cost * ncls + cls],
                            (unsigned long long)__double_as_longlong(acc));
              });
    __syncthreads();
    mix_visit(mt, C, need, S, tid, blockDim.x, my_flags,
              [&](uint32_t cost, uint32_t cls, double acc, uint64_t id) {
                  const uint64_t x = (uint64_t)cost * ncls + cls;
                  if ((uint64_t)__double_as_longlong(acc) == c_acc[x])
                      atomicMin((unsigned long long*)&c_id[x], (unsigned long long)id);
              });
    __syncthreads();

    // (b) exact dominance between cells: inclusive prefix maximum over (cost', class') <= (cost, class)
    for (uint32_t k = tid; k <= S; k += blockDim.x) {
        uint64_t run = 0;
        for (uint32_t l = 0; l < ncls; ++l) { const uint64_t a = c_acc[(uint64_t)k * ncls + l]; run = a > run ? a : run; c_pm[(uint64_t)k * ncls + l] = run; }
    }
    __syncthreads();
    for (uint32_t l = tid; l < ncls; l += blockDim.x) {
        uint64_t run = 0;
        for (uint32_t k = 0; k <= S; ++k) { const uint64_t a = c_pm[(uint64_t)k * ncls + l]; run = a > run ? a : run; c_pm[(uint64_t)k * ncls + l] = run; }
    }
    __syncthreads();
    for (uint64_t x = tid; x < ncell; x += blockDim.x) {
        const uint64_t a = c_acc[x];
        if (a == 0) continue;
        const uint32_t k = (uint32_t)(x / ncls), l = (uint32_t)(x % ncls);
        const uint64_t up = k > 0 ? c_pm[x - ncls] : 0, left = l > 0 ? c_pm[x - 1] : 0;
        if ((up > left ? up : left) >= a) continue;         // something cheaper-or-equal and faster-or-equal is as accurate
        c_list[atomicAdd(&s_n, 1u)] = (uint32_t)x;
    }
    __syncthreads();
    const uint32_t n = s_n;

    // latency of the option kept in cell x, from its id
    auto lat_of = [&](uint64_t id) -> uint32_t {
        if (id < C) return s_lat[id];
        const uint64_t pair = (id - C) >> 16;
        return umax(s_lat[pair / C], s_lat[pair % C]);
    };
    // (c) thinning over a grid of latency and accuracy.  The survivors in the order
    // (latency, id) are cut into `bands` runs; a band of more than `per` options keeps those
    // at evenly spaced ranks of its order by (accuracy, id).  c_pm is free now: its first
    // half lists the kept cells, its second half holds the band of every survivor.
    uint32_t* kept = (uint32_t*)c_pm;
    uint32_t* band = kept + ncell;
    uint32_t bands = 1;
    while ((uint64_t)(bands + 1) * (bands + 1) <= cap) ++bands;
    const uint32_t per = cap / bands;                       // >= 2
    if (n > cap) {
        my_flags |= F_TRUNCATED;
        for (uint32_t j = tid; j < n; j += blockDim.x) {
            const uint64_t id = c_id[c_list[j]];
            const uint32_t l = lat_of(id);
            uint32_t rank = 0;
            for (uint32_t o = 0; o < n; ++o) {
                const uint64_t id2 = c_id[c_list[o]];
                const uint32_t l2 = lat_of(id2);
                rank += (l2 < l || (l2 == l && id2 < id)) ? 1u : 0u;
            }
            band[j] = (uint32_t)((uint64_t)rank * bands / n);
        }
        __syncthreads();
    }
    for (uint32_t j = tid; j < n; j += blockDim.x) {
        const uint32_t x = c_list[j];
        bool keep = true;
        if (n > cap) {
            const uint64_t a = c_acc[x], id = c_id[x];
            const uint32_t b = band[j];
            uint32_t rank = 0, size = 0;
            for (uint32_t o = 0; o < n; ++o) {
                if (band[o] != b) continue;
                ++size;
                const uint32_t y = c_list[o];
                const uint64_t a2 = c_acc[y];
                rank += (a2 < a || (a2 == a && c_id[y] < id)) ? 1u : 0u;
            }
            if (size > per) {
                // is rank == floor(j*(size-1)/(per-1)) for some j < per ?
                const uint64_t jj = ((uint64_t)rank * (per - 1) + (size - 2)) / (size - 1);
                keep = (jj < per) && ((jj * (size - 1)) / (per - 1) == rank);
            }
        }
        if (keep) kept[atomicAdd(&s_kept, 1u)] = x;
    }
    __syncthreads();
    // (d) ascending id; the entry carries both tuples and both replica counts
    const uint32_t K = s_kept;
    Entry* out = pl.entries + ((size_t)i * pl.t_max + t) * pl.k_max;
    for (uint32_t j = tid; j < K; j += blockDim.x) {
        const uint32_t x = kept[j];
        const uint64_t id = c_id[x];
        uint32_t pos = 0;
        for (uint32_t o = 0; o < K; ++o) pos += c_id[kept[o]] < id ? 1u : 0u;
        Entry e;
        e.cost = (uint32_t)(x / ncls);
        e.acc = __longlong_as_double((long long)c_acc[x]);
        e.key = 0;
        if (id < C) {
            e.lat = s_lat[id];
            e.choice = (uint32_t)id | (0xFFFFu << 16);
            e.rep = e.cost / s_units[id];
        } else {
            const uint64_t pair = (id - C) >> 16;
            const uint32_t c1 = (uint32_t)(pair / C), c2 = (uint32_t)(pair % C), m1 = (uint32_t)((id - C) & 0xFFFFu);
            const uint32_t m2 = (e.cost - m1 * s_units[c1]) / s_units[c2];
            e.lat = umax(s_lat[c1], s_lat[c2]);
            e.choice = c1 | (c2 << 16);
            e.rep = m1 | (m2 << 16);
        }
        out[pos] = e;
    }
    if (my_flags) atomicOr(&s_flags, my_flags);
    __syncthreads();
    if (tid == 0) {
        in->K[t] = K;
        const uint32_t f = s_flags | (K == 0 ? F_EMPTY : 0);
        if (f) atomicOr(&in->flags, f);
        if (f & F_TRUNCATED) atomicOr(&in->trunc_mask, 1u << t);
    }
}

// How the enumeration's blocks share the tiles.  Tiles can go out by index, without any
// atomic, in rounds - in round r block b takes the run of OWN tiles that starts at
// (r * blocks + b) * OWN, so that all blocks move through the tile order together - or through
// one global counter, in batches.  Measured on the 20^8 sweep and on the batch of graphs:
//  * Atomics on one address go through one at a time, about 10 ns each.  A search with few
//    tiles per block spends longer waiting for tickets than working: it is shared out by
//    index alone.
//  * When every candidate is scored, tiles of one instance cost the same, but equal shares by
//    index still end unevenly: with 7 waves on a SIMD the vector ALU is saturated by about 5
//    and the waves launched last get what is left, so they finish their equal share late and
//    alone (34 ms with the counter against 47 ms by index on a quarter of the sweep).  There
//    the counter hands out everything, in 128 batches per block.
//  * With bounds, most tiles are excluded at once and the counter itself is the limit (tens
//    of tickets per microsecond): a quarter goes out by index and the rest in 8 batches per
//    block (9.1 ms against 16.6 ms for the sweep).
// Giving every block one long contiguous run was tried too and is slower still: seven blocks of
// a compute unit then stream seven instances' tables through one scalar cache.
constexpr uint32_t SEED_MIN_TILES_PER_BLOCK = 8;      // the plan kernel seeds the cost bound of instances from here on
constexpr uint32_t STATIC_ONLY_TILES_PER_BLOCK = 8;   // up to here: no counter at all
constexpr uint32_t BOUNDED_COUNTER_TILES_PER_BLOCK = 64;   // with bounds: below this no counter either (one level of a
                                                      // large search: 0.51-0.72 ms by index, 0.59-0.85 ms with tickets)
constexpr uint32_t ROUNDS_WANTED = 64;                // with bounds: rounds the part shared out by index is cut into
constexpr uint32_t BATCHES_PER_BLOCK_PLAIN = 128;     // batches per block from the counter, every candidate scored
constexpr uint32_t BATCHES_PER_BLOCK_BOUNDED = 8;     // ... and with bounds

// ---- plan -------------------------------------------------------------------------------
// Balancing of the tile sizes (scan_tiles): the enumeration's blocks should each see about this
// many tiles, but no tile is cut below MIN_TILE_COST candidates per lane, where the per-tile
// set-up would start to show.
constexpr uint32_t TILES_PER_BLOCK_WANTED = 16;
constexpr uint32_t MIN_TILE_COST = 2048;

__device__ __forceinline__ uint32_t bits_of(uint64_t x) { return x ? 64u - (uint32_t)__builtin_clzll(x) : 0u; }

// Exclusive prefix sum of a[0..n) (n <= 256 * 8) in place, by all 256 threads of the block;
// returns the total.  s_part: 256 words of scratch.
__device__ uint32_t block_exclusive_scan(uint32_t* a, uint32_t n, uint32_t* s_part)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t per = (n + 255) / 256;
    const uint32_t lo = tid * per, hi = lo + per < n ? lo + per : n;
    uint32_t sum = 0;
    for (uint32_t k = lo; k < hi; ++k) sum += a[k];
    s_part[tid] = sum;
    __syncthreads();
    for (uint32_t off = 1; off < 256; off <<= 1) {      // inclusive scan of the 256 partial sums
        const uint32_t v = tid >= off ? s_part[tid - off] : 0u;
        __syncthreads();
        s_part[tid] += v;
        __syncthreads();
    }
    uint32_t run = s_part[tid] - sum;
    const uint32_t total = s_part[255];
    for (uint32_t k = lo; k < hi; ++k) { const uint32_t v = a[k]; a[k] = run; run += v; }
    __syncthreads();
    return total;
}

// Exclusive prefix of v over the 256 threads of the block, and the total.  s: 256 words of scratch.
__device__ uint64_t block_scan_u64(uint64_t v, uint64_t* s, uint64_t* total)
{
    const uint32_t tid = threadIdx.x;
    s[tid] = v;
    __syncthreads();
    for (uint32_t off = 1; off < 256; off <<= 1) {
        const uint64_t x = tid >= off ? s[tid - off] : 0;
        __syncthreads();
        s[tid] += x;
        __syncthreads();
    }
    const uint64_t incl = s[tid];
    *total = s[255];
    __syncthreads();
    return incl - v;
}

// Run by the last plan block to finish: the global view.  Tiles that are much larger than the
// average share of a block are cut into smaller ones (fewer digits of the outermost in-lane
// loop per tile), so that blocks end together also when a few instances hold most of the work;
// then the exclusive scan of the tile counts, the total, and the counters' reset.
__device__ void scan_tiles(const Plan& pl, uint64_t* s_sum)
{
    const uint32_t tid = threadIdx.x, n = pl.n_inst;
    const uint32_t per = (n + 255) / 256;
    const uint32_t lo = tid * per, hi = (lo + per < n) ? lo + per : n;
    const volatile Instance* inst = pl.inst;          // written by other blocks
    uint64_t work = 0;
    for (uint32_t k = lo; k < hi; ++k) {
        const uint32_t tiles = inst[k].tiles, cost = inst[k].tile_cost;      // independent loads, one round trip
        work += (uint64_t)tiles * cost;
    }
    uint64_t total_work;
    (void)block_scan_u64(work, s_sum, &total_work);
    uint64_t target = total_work / ((uint64_t)pl.grid * TILES_PER_BLOCK_WANTED);
    if (target < MIN_TILE_COST) target = MIN_TILE_COST;
    uint64_t sum = 0;
    for (uint32_t k = lo; k < hi; ++k) {
        Instance* in = pl.inst + k;
        uint32_t tiles = inst[k].tiles, cost = inst[k].tile_cost;
        const uint32_t chunk = inst[k].chunk, unit = inst[k].unit_cost;
        if (tiles != 0 && inst[k].splittable && cost > target && chunk > 1) {
            uint64_t c = target / (unit ? unit : 1u);           // digits per tile that stay within the target
            if (c < 1) c = 1;
            if (c < chunk) {
                const uint32_t ko = inst[k].ko, n_chunks = (ko + (uint32_t)c - 1) / (uint32_t)c;
                if ((uint64_t)inst[k].n_groups * n_chunks <= 0x7FFFFFFFull) {
                    const uint64_t tc = c * unit;
                    cost = tc > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)tc;
                    tiles = inst[k].n_groups * n_chunks;
                    in->chunk = (uint32_t)c; in->n_chunks = n_chunks;
                    in->tiles = tiles; in->tile_cost = cost;
                }
            }
        }
        sum += tiles;
    }
    uint64_t total_tiles;
    uint64_t run = block_scan_u64(sum, s_sum, &total_tiles);
    for (uint32_t k = lo; k < hi; ++k) { pl.inst[k].tile_begin = run; pl.tile_begin[k] = run; run += inst[k].tiles; }
    if (tid == 0) {
        pl.summary->total_tiles = total_tiles;
        pl.summary->done_count = 0;
        pl.summary->any_flags = 0;
        pl.summary->visited = 0;
        // A cost bound found in one tile helps the tiles that start after it: with only a few
        // tiles per block everything runs at once and the bookkeeping would be pure overhead.
        // (From 8 tiles per block it pays: one 20^8-candidate level takes 0.6-0.8 ms instead of 2.0.)
        const bool bounded = pl.bounds && total_tiles >= (uint64_t)pl.grid * BOUNDS_MIN_TILES_PER_BLOCK;
        pl.summary->bounded = bounded ? 1u : 0u;
        // Rounds of own runs, then batches of the rest from the counter (see above).
        const uint64_t G = pl.grid;
        uint64_t own = 1, rounds = 0, batch;
        if (total_tiles <= G * STATIC_ONLY_TILES_PER_BLOCK || (bounded && total_tiles < G * BOUNDED_COUNTER_TILES_PER_BLOCK)) {
            rounds = (total_tiles + G - 1) / G; batch = 0;
        }
        else {
            if (bounded) {
                own = total_tiles / (4 * G * ROUNDS_WANTED);
                if (own < 1) own = 1;
                if (own > 0x40000000ull) own = 0x40000000ull;
                rounds = total_tiles / 4 / (G * own);
            }
            batch = (total_tiles - rounds * G * own) / (G * (bounded ? BATCHES_PER_BLOCK_BOUNDED : BATCHES_PER_BLOCK_PLAIN));
            if (batch < 1) batch = 1;
            if (batch > 0x40000000ull) batch = 0x40000000ull;
        }
        pl.summary->own_tiles = (uint32_t)own;
        pl.summary->own_rounds = (uint32_t)rounds;               // (at most 8 or about 64)
        pl.summary->batch_tiles = (uint32_t)batch;
        const uint64_t first = rounds * G * own;                 // the counter starts behind the rounds
        pl.summary->next_tile = (unsigned long long)(first < total_tiles ? first : total_tiles);
        pl.summary->best_level = -1;
        pl.summary->max_demand = 0;
    }
}

// One block per instance: strides of the caller's index order, key packing, choice
// of how many positions a lane loops over, tile geometry, local keys and the stream
// of the innermost position, reset of the partials.  The last block to finish scans
// the tile counts (plan_done is zeroed by the prune kernel, which runs before).
//
struct Score { uint32_t latency; uint32_t cost; double accuracy; uint8_t mask; };     // mask: bit 0 Eq. 3, 1 Eq. 13, 2 Eq. 8
__device__ Score score_digits(const Graph* g, const Instance* in, const Entry* entries, uint32_t k_max,
                              const uint32_t* dig);

// Written for latency (one small instance is often all there is): every pass over the
// entries covers all tasks at once (one round trip to memory instead of one per task), the
// quads of the innermost stream are laid out by a parallel scan, and what only one thread
// can decide is kept short.
__global__ void __launch_bounds__(256) plan_kernel(Plan pl)
{
    const uint32_t i = blockIdx.x, tid = threadIdx.x;
    Instance* in = pl.inst + i;
    const Graph* g = pl.graphs + in->problem;
    const uint32_t T = g->T;
    __shared__ uint32_t s_maxcost[MAXT], s_mincost[MAXT], s_K[MAXT], s_off[MAXT + 1], s_lsT[MAXT], s_minxlat;
    __shared__ uint32_t s_bits, s_lb, s_nin, s_ls[3], s_chunk, s_nq, s_last, s_nvx;
    __shared__ unsigned long long s_xtop;
    __shared__ uint64_t s_stride[MAXT];
    // the innermost position's entries, staged once: variant, latency, cost, and the first
    // quad of the variant that starts at digit d
    __shared__ uint16_t s_xvar[MAXC];
    __shared__ uint32_t s_xlat[MAXC], s_xcost[MAXC], s_xq0[MAXC];
    __shared__ uint64_t s_yacc[MAXC];       // position 1's accuracies as bit patterns (runs of equal accuracy)
    __shared__ uint16_t s_zvar[MAXC];       // position 2's variants (runs of one variant)
    __shared__ uint64_t s_sum[256];
    __shared__ uint32_t s_part[256];
    // graph facts the single-thread section below needs, fetched by many threads at once
    __shared__ uint32_t s_task_at[MAXT], s_capacity, s_PB;
    if (tid < MAXT) {
        s_maxcost[tid] = 0; s_mincost[tid] = 0xFFFFFFFFu; s_K[tid] = tid < T ? in->K[tid] : 0; s_lsT[tid] = 0xFFFFFFFFu;
        in->kmagic[tid] = magic_of(s_K[tid]);
        s_task_at[tid] = g->task_at[tid];
    }
    if (tid == 32) s_capacity = g->capacity;
    if (tid == 33) s_PB = g->P * g->B;
    if (tid == 0) s_minxlat = 0xFFFFFFFFu;
    __syncthreads();
    if (tid == 0) { uint32_t run = 0; for (uint32_t t = 0; t < T; ++t) { s_off[t] = run; run += s_K[t]; } s_off[T] = run; }
    if (tid >= 64 && tid < 64 + MAXT) {
        const uint32_t p = tid - 64, t = s_task_at[p];
        in->kpos[p] = p < T ? s_K[t] : 0;
        in->mpos[p] = magic_of(p < T ? s_K[t] : 0);
        in->rowpos[p] = p < T ? t * pl.k_max : 0;
    }
    if (tid == 96) { in->sloq = in->slo_l / g->q; in->pad_sloq = 0; }
    __syncthreads();
    const uint32_t tx = s_task_at[0], PB = s_PB, KX = s_K[tx], n_all = s_off[T];
    const Entry* ent = pl.entries + (size_t)i * pl.t_max * pl.k_max;
    // pass 1, all tasks at once: cost range per task; the innermost position's entries staged
    for (uint32_t f = tid; f < n_all; f += blockDim.x) {
        uint32_t t = 0;
        while (t + 1 < T && s_off[t + 1] <= f) ++t;
        const uint32_t d = f - s_off[t];
        const Entry* e = ent + (size_t)t * pl.k_max + d;
        const uint32_t c = e->cost;
        atomicMax(&s_maxcost[t], c);
        atomicMin(&s_mincost[t], c);
        if (t == tx) {
            const uint32_t lat = e->lat;
            s_xcost[d] = c; s_xlat[d] = lat; s_xvar[d] = (uint16_t)(e->choice / PB);
            atomicMin(&s_minxlat, lat);
        }
        if (T >= 2 && t == s_task_at[1]) s_yacc[d] = __builtin_bit_cast(uint64_t, e->acc);
        if (T >= 3 && t == s_task_at[2]) s_zvar[d] = (uint16_t)(e->choice / PB);
    }
    __syncthreads();
    // quads of position 0's stream (single tuples): every variant's entries rounded up to whole
    // quads.  The first digit of a variant counts its entries; an exclusive scan places it.
    for (uint32_t d = tid; d < KX; d += blockDim.x) {
        uint32_t q = 0;
        if (d == 0 || s_xvar[d - 1] != s_xvar[d]) {
            const uint32_t var = s_xvar[d];
            uint32_t d1 = d + 1;
            while (d1 < KX && s_xvar[d1] == var) ++d1;
            q = (d1 - d + 3) / 4;
        }
        s_xq0[d] = q;
    }
    __syncthreads();
    const uint32_t nq_groups = block_exclusive_scan(s_xq0, KX, s_part);
    if (tid == 0) {
        uint64_t space = 1, cost_bound = 0;
        bool over = false;
        for (uint32_t t = 0; t < T; ++t) {
            s_stride[t] = space;
            in->stride[t] = space;
            const uint64_t k = s_K[t];
            if (k != 0 && __umul64hi(space, k) != 0) over = true;
            space *= k;
            cost_bound += s_maxcost[t];
        }
        if (space >> 63) over = true;
        const uint32_t idx_bits = space <= 1 ? 0u : bits_of(space - 1);
        const uint32_t cost_bits = bits_of(cost_bound);
        if (cost_bound > 0x7FFFFFFFull || idx_bits + cost_bits > 63) over = true;
        if (over) { space = 0; atomicOr(&in->flags, F_OVERFLOW); }
        in->space = space;
        in->idx_bits = idx_bits;
        // Eq. 8 for the whole instance: if even the cheapest entry of every task together exceeds
        // S_avail, no candidate fits and nothing needs to be enumerated (bounds on only).
        bool none_fits = false;
        if (pl.cut && s_capacity != 0 && space != 0) {
            uint64_t least = 0;
            for (uint32_t t = 0; t < T; ++t) least += s_mincost[t];
            none_fits = least > s_capacity;
            if (none_fits) atomicOr(&in->flags, F_CUT);
        }

        // how many leading positions a lane loops over, and the tile geometry
        uint32_t Kp[MAXT];
        for (uint32_t p = 0; p < T; ++p) Kp[p] = s_K[s_task_at[p]];
        uint32_t n_in = 1;
        uint64_t s_out = 0;
        const uint32_t n_top = T < 3 ? T : 3;
        if (space != 0) {
            for (uint32_t n = n_top; n >= 1; --n) {
                uint64_t so = 1;
                for (uint32_t p = n; p < T; ++p) so *= Kp[p];
                if (n == 1 || (so >= 64 && (so >= pl.lanes_wanted || so * Kp[n - 1] >= pl.lanes_wanted))) { n_in = n; s_out = so; break; }
            }
        }
        // 32-bit fast path: candidates of one lane-tile differ only in the in-lane positions,
        // so they can be ordered by (cost of those positions << lb) | rank, where rank orders
        // them as the caller's index does (in-lane task with the lowest id = least significant).
        uint32_t ord[3] = {0, 1, 2}, ls[3] = {0, 0, 0}, lb = 0, use32 = 0, nq = 0;
        if (space != 0) {
            for (uint32_t a = 0; a < n_in; ++a)           // sort in-lane positions by task id
                for (uint32_t b = a + 1; b < n_in; ++b)
                    if (s_task_at[ord[b]] < s_task_at[ord[a]]) { const uint32_t x = ord[a]; ord[a] = ord[b]; ord[b] = x; }
            uint64_t ranks = 1, cost_in = 0;
            for (uint32_t a = 0; a < n_in; ++a) {
                ls[ord[a]] = (uint32_t)ranks;
                ranks *= Kp[ord[a]];
                cost_in += s_maxcost[s_task_at[ord[a]]];
            }
            lb = bits_of(ranks - 1);
            const uint32_t cb = bits_of(cost_in);
            use32 = (ranks <= 0x7FFFFFFFull && lb + cb <= 31) ? 1u : 0u;
        }
        if (use32) nq = pl.mix ? (KX + 3) / 4 : nq_groups;      // mixtures: one stream in latency order
        uint32_t chunk = 1, n_chunks = 0, n_groups = 0, ko = 0;
        uint64_t inner = 1;
        const bool stream = use32 && n_in == 1;
        if (space != 0 && !none_fits) {
            // extent of the outermost in-lane loop: digits, or quads when it is the stream itself
            inner = stream ? 4 : 1;
            for (uint32_t p = 0; p + 1 < n_in; ++p) inner *= Kp[p];
            const uint32_t Ko = stream ? nq : Kp[n_in - 1];
            uint64_t c = s_out >= pl.lanes_wanted ? Ko : (s_out * Ko) / pl.lanes_wanted;   // extent per tile that
            if (c > Ko) c = Ko;                                          // still leaves lanes_wanted lanes busy
            const uint64_t c_min = (64 + inner - 1) / inner;             // at least 64 candidates per lane
            if (c < c_min) c = c_min;
            if (c > Ko) c = Ko;
            if (c < 1) c = 1;
            chunk = (uint32_t)c;
            ko = Ko;
            n_chunks = (Ko + chunk - 1) / chunk;
            const uint64_t ng = (s_out + TILE_LANES - 1) / TILE_LANES;
            if (ng * n_chunks > 0x7FFFFFFFull) { atomicOr(&in->flags, F_OVERFLOW); n_chunks = 0; }
            else n_groups = (uint32_t)ng;
        }
        in->n_in = n_in; in->s_out = s_out; in->chunk = chunk;
        in->n_chunks = n_chunks; in->n_groups = n_groups;
        in->tiles = n_groups * n_chunks;
        // what scan_tiles needs to rebalance: candidates per lane of one tile and of one digit of
        // its chunked loop (clamped), that loop's extent, and whether its cut may change (the
        // stream's quads carry flags that depend on the cut)
        const uint64_t tc = inner * chunk;
        in->unit_cost = inner > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)inner;
        in->tile_cost = tc > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)tc;
        in->ko = ko;
        in->splittable = stream ? 0u : 1u;
        in->use32 = use32; in->lb = lb; in->nq = nq;
        in->nvx = 0;                      // set with the stream of single tuples, if there is one
        in->pair_nq = 0;                  // set with the pair stream, if there is one
        s_nvx = 0;
        s_xtop = 0;
        uint64_t min_in = 0;
        for (uint32_t p = 0; p < n_in; ++p) min_in += s_mincost[s_task_at[p]];
        in->min_in_cost = (space != 0 && pl.bounds) ? (uint32_t)(min_in > 0xFFFFFFFFull ? 0xFFFFFFFFull : min_in) : 0u;
        in->min_x_lat = pl.bounds ? s_minxlat : 0u;
        in->min_x_cost = (space != 0 && pl.bounds) ? s_mincost[tx] : 0u;
        in->min_xy_cost = (space != 0 && pl.bounds && n_in >= 2) ? s_mincost[tx] + s_mincost[s_task_at[1]] : 0u;
        pl.bound[i] = s_capacity != 0 ? s_capacity : 0xFFFFFFFFu;
        pl.best_obj[i] = ordered_bits(-__builtin_inf());
        if (space != 0 && !use32) atomicOr(&in->flags, F_WIDE);
        for (int a = 0; a < 3; ++a) { in->ord[a] = ord[a]; s_ls[a] = ls[a]; }
        if (use32) for (uint32_t p = 0; p < n_in; ++p) s_lsT[s_task_at[p]] = ls[p];
        s_bits = idx_bits; s_lb = lb; s_nin = use32 ? n_in : 0;
        s_chunk = stream ? chunk : 0; s_nq = nq;
    }
    __syncthreads();
    // pass 2, all tasks at once: packed keys (cost << idx_bits) | digit * stride, and for the
    // in-lane positions the 32-bit local keys (cost << lb) | digit * local stride
    {
        const uint32_t idx_bits = s_bits, lb = s_lb;
        Entry* entw = pl.entries + (size_t)i * pl.t_max * pl.k_max;
        uint32_t* k32 = pl.k32 + (size_t)i * pl.t_max * pl.k_max;
        for (uint32_t f = tid; f < n_all; f += blockDim.x) {
            uint32_t t = 0;
            while (t + 1 < T && s_off[t + 1] <= f) ++t;
            const uint32_t d = f - s_off[t];
            Entry* e = entw + (size_t)t * pl.k_max + d;
            const uint32_t c = e->cost;
            e->key = ((uint64_t)c << idx_bits) | ((uint64_t)d * s_stride[t]);
            if (s_lsT[t] != 0xFFFFFFFFu) k32[(size_t)t * pl.k_max + d] = (c << lb) | (d * s_lsT[t]);
        }
    }
    // stream of position 0: by variant, inside a variant by ascending latency (so that the
    // lanes still feasible only shrink along a variant), each variant padded to whole quads
    if (s_nin != 0 && pl.mix) {
        // mixture mode: all entries in ascending latency, each with its own accuracy
        const Entry* ex = ent + (size_t)tx * pl.k_max;
        QuadM* qm = (QuadM*)(pl.quads + (size_t)i * quad_stride(pl.k_max));
        for (uint32_t d = tid; d < KX; d += blockDim.x) {
            const uint32_t lat = s_xlat[d];
            uint32_t rank = 0;
            for (uint32_t x = 0; x < KX; ++x) rank += (s_xlat[x] < lat || (s_xlat[x] == lat && x < d)) ? 1u : 0u;
            XEntM me;
            me.lat = lat; me.k32 = (s_xcost[d] << s_lb) | (d * s_ls[0]); me.acc = ex[d].acc;
            qm[rank / 4].e[rank % 4] = me;
        }
        // the most accurate option of position 0: a ceiling for objective mode (positive doubles order as their bits)
        {
            unsigned long long top = 0;
            for (uint32_t d = tid; d < KX; d += blockDim.x) {
                const unsigned long long b = __builtin_bit_cast(unsigned long long, ex[d].acc);
                top = b > top ? b : top;
            }
            if (top != 0) atomicMax(&s_xtop, top);
        }
        for (uint32_t r = KX + tid; r < s_nq * 4; r += blockDim.x) {
            XEntM pad;
            pad.lat = 0xFFFFFFFFu; pad.k32 = 0xFFFFFFFFu; pad.acc = 0.0;
            qm[r / 4].e[r % 4] = pad;
        }
        __syncthreads();
        if (tid == 0) in->xacc[0] = __builtin_bit_cast(double, s_xtop);
    } else if (s_nin != 0) {
        const Entry* ex = ent + (size_t)tx * pl.k_max;
        Quad* qd = pl.quads + (size_t)i * quad_stride(pl.k_max);
        QuadC* qc = (QuadC*)(qd + quadc_offset(pl.k_max));
        for (uint32_t d = tid; d < KX; d += blockDim.x) {
            const uint32_t var = s_xvar[d], lat = s_xlat[d];
            uint32_t d0 = d, d1 = d + 1, rank = 0;
            while (d0 > 0 && s_xvar[d0 - 1] == var) --d0;
            while (d1 < KX && s_xvar[d1] == var) ++d1;
            for (uint32_t x = d0; x < d1; ++x) rank += (s_xlat[x] < lat || (s_xlat[x] == lat && x < d)) ? 1u : 0u;
            const uint32_t q0 = s_xq0[d0], n = d1 - d0, quads = (n + 3) / 4;
            XEnt me;
            me.lat = lat;
            me.k32 = (s_xcost[d] << s_lb) | (d * s_ls[0]);
            qd[q0 + rank / 4].e[rank % 4] = me;
            qc[q0 + rank / 4].e[rank % 4] = me;
            if (d == d0) {                                   // the variant's first digit writes headers and padding
                const double acc = ex[d].acc;
                for (uint32_t j = 0; j < quads; ++j) {
                    qd[q0 + j].acc = acc;
                    // the accuracy test is (re)done where a variant starts and where a tile's range starts
                    qd[q0 + j].newgrp = (j == 0 || (s_chunk != 0 && (q0 + j) % s_chunk == 0)) ? 1u : 0u;
                    for (int z = 0; z < 5; ++z) qd[q0 + j].pad[z] = 0;
                }
                for (uint32_t r = n; r < quads * 4; ++r) {
                    XEnt pad;
                    pad.lat = 0xFFFFFFFFu; pad.k32 = 0xFFFFFFFFu;
                    qd[q0 + r / 4].e[r % 4] = pad;
                    qc[q0 + r / 4].e[r % 4] = pad;
                }
                // the variant's place in the stream, and its accuracy for the waves that keep
                // one accuracy mask per variant
                uint32_t ordinal = 0;
                for (uint32_t x = 1; x <= d0; ++x) ordinal += s_xvar[x - 1] != s_xvar[x] ? 1u : 0u;
                if (ordinal < (uint32_t)MAX_XVAR) { in->xacc[ordinal] = acc; in->xqe[ordinal] = (q0 + quads) * (uint32_t)sizeof(QuadC); }
                if (d1 == KX) {
                    in->nvx = ordinal + 1;
                    s_nvx = ordinal + 1;
                    for (uint32_t v = ordinal + 1; v < (uint32_t)MAX_XVAR; ++v) in->xqe[v] = (q0 + quads) * (uint32_t)sizeof(QuadC);
                }
            }
        }
    }
    // position 1's digits for the loop that batches them (single tuples, two or more in-lane positions)
    if (s_nin >= 2 && !pl.mix) {
        const uint32_t ty = s_task_at[1], KY = s_K[ty];
        const Entry* ey = ent + (size_t)ty * pl.k_max;
        uint32_t* ylat = (uint32_t*)(pl.quads + (size_t)i * quad_stride(pl.k_max) + yrec_offset(pl.k_max));
        uint32_t* yk32 = ylat + ydigit_words(pl.k_max);
        uint32_t* yrun = yk32 + ydigit_words(pl.k_max);
        for (uint32_t d = tid; d < KY; d += blockDim.x) {
            const uint64_t bits = s_yacc[d];
            uint32_t e = d + 1;
            while (e < KY && s_yacc[e] == bits) ++e;
            ylat[d] = ey[d].lat; yk32[d] = (ey[d].cost << s_lb) | (d * s_lsT[ty]); yrun[d] = e;
        }
        if (pl.bounds) {
            // for the bounds: the smallest key and the lowest latency from each digit to the end of its run
            uint32_t* yrk = yrun + 2 * ydigit_words(pl.k_max);
            uint32_t* yrl = yrk + ydigit_words(pl.k_max);
            for (uint32_t d = tid; d < KY; d += blockDim.x) {
                const uint64_t bits = s_yacc[d];
                uint32_t mk = 0xFFFFFFFFu, ml = 0xFFFFFFFFu;
                for (uint32_t x = d; x < KY && s_yacc[x] == bits; ++x) {
                    mk = umin(mk, (ey[x].cost << s_lb) | (x * s_lsT[ty]));
                    ml = umin(ml, ey[x].lat);
                }
                yrk[d] = mk; yrl[d] = ml;
            }
        }
        if (s_nin >= 3) {
            // position 2: per digit the end of its run of one variant
            uint32_t* zrun = yrun + ydigit_words(pl.k_max);
            const uint32_t KZ = s_K[s_task_at[2]];
            for (uint32_t d = tid; d < KZ; d += blockDim.x) {
                const uint16_t var = s_zvar[d];
                uint32_t e = d + 1;
                while (e < KZ && s_zvar[e] == var) ++e;
                zrun[d] = e;
            }
        }
    }
    // pair stream (three in-lane positions, single tuples, few variants in position 0): per digit
    // of position 1 the records of position 0's stream with that digit's local key added to
    // every key.  Built from what this block has just written (read back past the L1).
    if (s_nin >= 3 && !pl.mix) {
        __syncthreads();
        const uint32_t nq = s_nq, KY = s_K[s_task_at[1]];
        const bool fits = pl.pair_cap != 0 && s_nvx >= 1 && s_nvx <= (uint32_t)MAX_XVAR && (uint64_t)nq * KY <= pl.pair_cap;
        if (fits) {
            const uint32_t* xw = (const uint32_t*)(pl.quads + (size_t)i * quad_stride(pl.k_max) + quadc_offset(pl.k_max));
            const uint32_t* yk = (const uint32_t*)(pl.quads + (size_t)i * quad_stride(pl.k_max) + yrec_offset(pl.k_max)) +
                                 ydigit_words(pl.k_max);
            XEnt* pr = (XEnt*)(pl.pairs + (size_t)i * (pl.pair_cap + 1));
            const uint32_t per = nq * 4;
            for (uint32_t f = tid; f < KY * per; f += blockDim.x) {
                const uint32_t dy = f / per, e = f % per;
                XEnt me;
                me.lat = __hip_atomic_load(xw + 2 * e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const uint32_t kx = __hip_atomic_load(xw + 2 * e + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const uint32_t ky = __hip_atomic_load(yk + dy, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                me.k32 = kx == 0xFFFFFFFFu ? kx : kx + ky;          // padding stays padding
                pr[f] = me;
            }
            if (tid < 4) { XEnt pad; pad.lat = 0xFFFFFFFFu; pad.k32 = 0xFFFFFFFFu; pr[KY * per + tid] = pad; }
            if (tid == 0) in->pair_nq = nq;
        }
    }
    // A first cost bound for the search with bounds (cost modes): steepest descent over single-task
    // swaps, from the most accurate choice of every task (fastest, then cheapest among equals).
    // Every step takes the swap that saves most among those that keep Eq. 3, 8 and 13, each scored
    // as the finalize kernel scores the winner; what it ends on is a candidate of the searched
    // space that meets all three, so its cost is a bound the optimum cannot exceed (candidates as
    // cheap as the bound stay in).  The enumeration otherwise starts every instance against
    // S_avail and finds the cheap candidates only where its loops happen to reach them.  The
    // descent takes some tens of microseconds (a few dozen rounds of scoring from global memory),
    // so it runs for instances with enough tiles to win that back.
    if (pl.bounds && !pl.objective && in->tiles >= SEED_MIN_TILES_PER_BLOCK * pl.grid) {
        __shared__ uint32_t s_dig[MAXT], s_seed_cost, s_seed_ok;
        __shared__ unsigned long long s_swap;
        const Entry* ent = pl.entries + (size_t)i * pl.t_max * pl.k_max;
        __syncthreads();
        if (tid < T) {
            const Entry* row = ent + (size_t)tid * pl.k_max;
            uint32_t bd = 0;
            for (uint32_t d = 1; d < s_K[tid]; ++d) {
                const Entry& e = row[d];
                const Entry& b = row[bd];
                if (e.acc > b.acc || (e.acc == b.acc && (e.lat < b.lat || (e.lat == b.lat && e.cost < b.cost)))) bd = d;
            }
            s_dig[tid] = bd;
        }
        __syncthreads();
        uint32_t dig[MAXT];
        for (uint32_t t = 0; t < MAXT; ++t) dig[t] = t < T ? s_dig[t] : 0;
        if (tid == 0) {
            const Score sc = score_digits(g, in, ent, pl.k_max, dig);
            s_seed_ok = (sc.mask == 7 && sc.cost < 0x7FFFFFFFu) ? 1u : 0u;     // (the scorer clamps costs there)
            s_seed_cost = sc.cost;
        }
        __syncthreads();
        const bool seeded = s_seed_ok != 0;
        for (uint32_t it = 0; seeded && it < 64; ++it) {
            if (tid == 0) s_swap = 0;
            __syncthreads();
            unsigned long long mine = 0;
            for (uint32_t f = tid; f < n_all; f += blockDim.x) {
                uint32_t t = 0;
                while (t + 1 < T && s_off[t + 1] <= f) ++t;
                const uint32_t d = f - s_off[t], old = dig[t];
                const uint32_t c_old = ent[(size_t)t * pl.k_max + old].cost, c_new = ent[(size_t)t * pl.k_max + d].cost;
                if (c_new >= c_old) continue;
                dig[t] = d;
                const Score sc = score_digits(g, in, ent, pl.k_max, dig);
                dig[t] = old;
                if (sc.mask == 7) {
                    const unsigned long long k = ((unsigned long long)(c_old - c_new) << 32) | (0xFFFFFFFFu - f);
                    mine = k > mine ? k : mine;
                }
            }
            if (mine != 0) atomicMax(&s_swap, mine);
            __syncthreads();
            const unsigned long long won = s_swap;
            if (won == 0) break;
            const uint32_t f = 0xFFFFFFFFu - (uint32_t)won;
            uint32_t t = 0;
            while (t + 1 < T && s_off[t + 1] <= f) ++t;
            dig[t] = f - s_off[t];
            if (tid == 0) s_seed_cost -= (uint32_t)(won >> 32);
            __syncthreads();
        }
        if (tid == 0 && seeded) atomicMin(pl.bound + i, s_seed_cost);
    }
    for (uint32_t b = tid; b < pl.grid; b += blockDim.x) {
        pl.partial[(size_t)i * pl.grid + b] = NO_KEY;
        pl.partial_obj[(size_t)i * pl.grid + b] = -__builtin_inf();
    }
    // last block: tile scan
    __threadfence();
    __syncthreads();
    if (tid == 0) s_last = (atomicAdd(&pl.summary->plan_done, 1u) == pl.n_inst - 1) ? 1u : 0u;
    __syncthreads();
    if (s_last) { __threadfence(); scan_tiles(pl, s_sum); }
}

// ---- enumeration ------------------------------------------------------------------------
// State a lane carries into the loops over positions 0..NIN-1: for each of those
// positions the part of its recursion that comes from positions >= NIN, plus what
// the sources among the outer positions already contribute.
struct LaneState {
    uint32_t nxt[3];    // max tail over successors seen so far
    double   hin[3];    // sum of w * H over successors seen so far
    uint32_t smax;      // max tail over sources seen so far
    double   sacc;      // sum of H over sources seen so far
    uint64_t key;       // sum of the 64-bit keys of the fixed positions
    uint32_t k32;       // sum of the 32-bit local keys of the fixed in-lane positions
    uint32_t cost_out;  // cost of the positions outside the lane loops (objective mode)
};

struct Uniforms {       // wave-uniform facts about positions 0..2
    const Entry JSV_CONST* tab[3];
    const uint32_t JSV_CONST* k32[3];
    const Quad JSV_CONST* quads;
    uint32_t K[3];
    bool     src[3];
    uint32_t m01, m02, m12;   // all ones if position a has an edge to position b, else 0
    double   w01, w02, w12;   // share of a among the predecessors of b (0 if no edge)
    uint32_t sloq;      // floor(SLO_l / q)
    uint32_t min_x_lat; // lowest latency of position 0's entries: below it a lane has no candidate
    uint32_t min_x_cost; // cheapest entry of position 0
    uint32_t min_xy_cost; // cheapest entries of positions 0 and 1 together
    uint32_t bound;     // total cost beyond which a candidate cannot be the answer (as known when the tile's loops start)
    uint32_t* bound_at; // where the instance's bound lives (with bounds: read and lowered while a tile runs)
    unsigned long long* best_obj_at;    // objective mode: likewise the best objective reached (ordered bit pattern)
    double   obj_seen;  // objective mode: an objective some wave has already reached for this instance (-inf: none known)
    double   slo_raw;   // SLO_a * A_max
    // objective mode (Eq. 14)
    uint32_t idx_bits, lb, capacity;
    double   alpha_n, beta;   // objective = alpha_n * A_raw - beta * cost
    double   alpha, inv_beta; // for the cost beyond which an objective already reached is out of reach; inv_beta 0: no such limit
    bool     mix;             // entries carry their own accuracies (mixtures)
    // single tuples: variants in position 0's stream and their accuracies (see loop_y_masked)
    uint32_t nvx;
    const double JSV_CONST* xacc;
    const uint32_t JSV_CONST* xqe;     // where each variant ends in the QuadC copy of the stream (bytes)
    const QuadC JSV_CONST* xq;         // that copy
    const uint32_t JSV_CONST* ylat;    // position 1's digits: latencies,
    const uint32_t JSV_CONST* yk32;    // local keys,
    const uint32_t JSV_CONST* yrun;    // ends of their runs of equal accuracy
    const uint32_t JSV_CONST* zrun;    // position 2's digits: ends of their runs of one variant
    const uint32_t JSV_CONST* yrk;     // position 1's digits: smallest local key and
    const uint32_t JSV_CONST* yrl;     // lowest latency from the digit to the end of its run (with bounds only)
    const QuadC JSV_CONST* pairs;      // pair stream: per digit of position 1, position 0's records with that digit's key added
    uint32_t pair_nq;                  // records per digit in it; 0: none
};

// Fix position P (a wave-uniform entry) and push its contribution down.  hin[P]
// already holds the sink share u(P) when P is a sink (it then has no successor),
// and an absent edge has weight 0 and mask 0, so only the "is a source" test is a
// (wave-uniform) branch.
template <int P>
__device__ __forceinline__ LaneState fix_position(const LaneState& s, const Uniforms& U,
                                                  uint32_t lat, double acc, uint64_t key, uint32_t k32)
{
#pragma clang fp contract(off)      // the product below is rounded on its own (see jsv_device.h)
    LaneState r = s;
    const uint32_t tail = lat + s.nxt[P];
    const double H = acc * s.hin[P];
    r.key = s.key + key;
    r.k32 = s.k32 + k32;
    if (U.src[P]) {
        asm volatile("" ::: "memory");      // rare (a source after position 0): keep it a real, wave-uniform branch
        r.smax = umax(s.smax, tail); r.sacc = s.sacc + H;
    }
    if constexpr (P == 2) {
        r.nxt[1] = umax(s.nxt[1], tail & U.m12); r.hin[1] = __builtin_fma(U.w12, H, s.hin[1]);
        r.nxt[0] = umax(s.nxt[0], tail & U.m02); r.hin[0] = __builtin_fma(U.w02, H, s.hin[0]);
    }
    if constexpr (P == 1) {
        r.nxt[0] = umax(s.nxt[0], tail & U.m01); r.hin[0] = __builtin_fma(U.w01, H, s.hin[0]);
    }
    return r;
}

// Innermost loop: position 0 (always a source, all its successors fixed).  Every
// candidate gets its latency compare (Eq. 3, against a hoisted threshold), its
// accuracy (Eq. 11-12) and compare (Eq. 13), its key, and the running minimum.
// The capacity bound (Eq. 8) is applied to the minimum afterwards: the cheapest
// candidate meeting Eq. 3 and 13 exceeds S_avail exactly when every such
// candidate does.
//
// 64-bit form: the full (cost, index) key per candidate.
template <bool BOUNDS>
__device__ __forceinline__ void loop_x64(const LaneState& s, const Uniforms& U, uint32_t lo, uint32_t hi,
                                         uint64_t& best, uint32_t& visits)
{
    const uint32_t worst = umax(s.smax, s.nxt[0]);           // dead lanes carry smax = 0xFFFFFFFF
    uint32_t thr = worst <= U.sloq ? U.sloq - s.nxt[0] : 0u;         // latencies are >= 1
    if constexpr (BOUNDS) {
        if ((s.key >> U.idx_bits) + U.min_x_cost > U.bound) thr = 0;    // too costly whatever position 0 takes
        if (__builtin_amdgcn_ballot_w64(thr >= U.min_x_lat) == 0) return;   // no lane of the wave has a candidate here
    }
    if (BOUNDS || U.mix) visits += hi - lo;
    const double cx = s.hin[0];
    const Entry JSV_CONST* tx = U.tab[0];
    for (uint32_t d = lo; d < hi; ++d) {
        const uint32_t lat = tx[d].lat;
        const double acc = tx[d].acc;
        const uint64_t k = s.key + tx[d].key;
        const bool ok = (lat <= thr) & (__builtin_fma(acc, cx, s.sacc) >= U.slo_raw);
        best = (ok && k < best) ? k : best;
    }
}

// 32-bit form.  Entries come as quads of one variant, inside a variant in ascending
// latency.  The accuracy of Eq. 11-13 is evaluated once per variant and its outcome
// becomes the execution mask (v_cmpx_le_f64); along the variant's candidates
// v_cmpx_le_u32 narrows the mask to the lanes that also meet the latency threshold
// of Eq. 3 - a lane that fails one candidate fails all later ones of the variant -
// and v_min_u32 updates the running minimum of 32-bit local keys of the lanes still
// in the mask.  Per candidate: two vector instructions and no scalar one.
//
// The whole loop is one asm block so that nothing else executes under the narrowed
// mask: one 64-byte scalar load per quad into s[72:87] (entries in dwords 0-7,
// accuracy in 8-9, new-variant flag in 10), byte offset in s88.  `full` is the
// execution mask of the surrounding convergent code; it is put back before the
// block ends, and the trailing s_nop keeps a following v_readlane /
// v_readfirstlane clear of the last vector write to EXEC.  The range [qlo, qhi) is
// never empty and its first quad always carries the new-variant flag.
template <bool BOUNDS>
__device__ __forceinline__ void loop_x32(const LaneState& s, const Uniforms& U, uint32_t qlo, uint32_t qhi,
                                         uint64_t full, uint32_t& best32, uint32_t& visits)
{
    // lanes whose other sources already break the latency SLO sit out (dead lanes carry
    // smax = 0xFFFFFFFF); for the rest position 0 may take at most thr (latencies are >= 1).
    // A lane whose thr is below every latency of position 0 has no candidate here; if that
    // holds for the whole wave the loop is skipped.
    const uint32_t thr = __builtin_elementwise_sub_sat(U.sloq, s.nxt[0]);
    uint64_t alive;
    if constexpr (BOUNDS) {
        // also out: lanes whose fixed positions plus the cheapest entry here cost more than the bound
        const uint32_t fixed = s.cost_out + (s.k32 >> U.lb);
        alive = __builtin_amdgcn_ballot_w64((s.smax <= U.sloq) & (thr >= U.min_x_lat) & (fixed + U.min_x_cost <= U.bound));
    } else alive = __builtin_amdgcn_ballot_w64(s.smax <= U.sloq);
    if (BOUNDS && alive == 0) return;
    if constexpr (BOUNDS) visits += (qhi - qlo) * 4u;
    uint32_t m = 0xFFFFFFFFu;
    double t;
#if defined(__HIP_DEVICE_COMPILE__)
    // SKIP: with bounds on, a quad whose fastest candidate no lane can take (or whose variant
    // no lane's accuracy allows) is left at once: the mask is already empty for its rest.
#define JSV_X32_LOOP(SKIP)                                                                         \
    asm volatile(                                                                                  \
        "s_mov_b32 s88, %[begin]\n\t"                                                              \
        "1:\n\t"                                                                                   \
        "s_load_dwordx16 s[72:87], %[base], s88\n\t"                                               \
        "s_add_u32 s88, s88, 64\n\t"                                                               \
        "s_waitcnt lgkmcnt(0)\n\t"                                                                 \
        "s_cmp_eq_u32 s82, 0\n\t"                                                                  \
        "s_cbranch_scc1 2f\n\t"                                                                    \
        "s_mov_b64 exec, %[alive]\n\t"                                                             \
        "v_fma_f64 %[t], s[80:81], %[cx], %[sacc]\n\t"                                             \
        "v_cmpx_le_f64_e32 vcc, %[slo], %[t]\n\t"                                                  \
        "2:\n\t"                                                                                   \
        "v_cmpx_le_u32_e32 vcc, s72, %[thr]\n\t"                                                   \
        SKIP                                                                                       \
        "v_min_u32_e32 %[m], s73, %[m]\n\t"                                                        \
        "v_cmpx_le_u32_e32 vcc, s74, %[thr]\n\t"                                                   \
        "v_min_u32_e32 %[m], s75, %[m]\n\t"                                                        \
        "v_cmpx_le_u32_e32 vcc, s76, %[thr]\n\t"                                                   \
        "v_min_u32_e32 %[m], s77, %[m]\n\t"                                                        \
        "v_cmpx_le_u32_e32 vcc, s78, %[thr]\n\t"                                                   \
        "v_min_u32_e32 %[m], s79, %[m]\n\t"                                                        \
        "4:\n\t"                                                                                   \
        "s_cmp_lt_u32 s88, %[end]\n\t"                                                             \
        "s_cbranch_scc1 1b\n\t"                                                                    \
        "s_mov_b64 exec, %[full]\n\t"                                                              \
        "s_nop 1"                                                                                  \
        : [m] "+v"(m), [t] "=&v"(t)                                                                \
        : [base] "s"(U.quads), [begin] "s"(qlo * 64u), [end] "s"(qhi * 64u), [full] "s"(full),     \
          [alive] "s"(alive),                                                                      \
          [thr] "v"(thr), [cx] "v"(s.hin[0]), [sacc] "v"(s.sacc), [slo] "s"(U.slo_raw)             \
        : "vcc", "scc", "s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", "s80", "s81", "s82", \
          "s83", "s84", "s85", "s86", "s87", "s88")
    if constexpr (BOUNDS) { JSV_X32_LOOP("s_cbranch_execz 4f\n\t"); }
    else { JSV_X32_LOOP(""); }
#undef JSV_X32_LOOP
#else
    (void)thr; (void)t; (void)qlo; (void)qhi; (void)full; (void)alive;
#endif
    const uint32_t cand = __builtin_elementwise_add_sat(s.k32, m);   // stays 0xFFFFFFFF if none
    best32 = best32 < cand ? best32 : cand;
}

// Mixture mode, 32-bit form.  Every entry carries its own accuracy; the stream is in ascending
// latency, so the latency compare narrows the execution mask for good (and ends the loop
// once no lane is left), while the accuracy compare masks one candidate only: the mask is
// saved before it and put back after the minimum.  Per candidate four vector instructions
// (latency compare, fma, accuracy compare, minimum) and two scalar moves.  A quad is one
// 64-byte scalar load into s[72:87]: per entry latency, local key, accuracy (2 dwords).
template <bool BOUNDS>
__device__ __forceinline__ void loop_x32_mix(const LaneState& s, const Uniforms& U, uint32_t qlo, uint32_t qhi,
                                             uint64_t full, uint32_t& best32, uint32_t& visits)
{
    const uint32_t thr = __builtin_elementwise_sub_sat(U.sloq, s.nxt[0]);
    uint64_t alive;
    if constexpr (BOUNDS) {
        // also out: lanes whose fixed positions plus the cheapest entry here cost more than the bound
        const uint32_t fixed = s.cost_out + (s.k32 >> U.lb);
        alive = __builtin_amdgcn_ballot_w64((s.smax <= U.sloq) & (thr >= U.min_x_lat) & (fixed + U.min_x_cost <= U.bound));
    } else alive = __builtin_amdgcn_ballot_w64(s.smax <= U.sloq);
    if (BOUNDS && alive == 0) return;
    uint32_t m = 0xFFFFFFFFu, pos = qhi * 64u;
    double t;
#if defined(__HIP_DEVICE_COMPILE__)
#define JSV_MIX_ENTRY(LAT, KEY, ACC)                       \
        "v_cmpx_le_u32_e32 vcc, " LAT ", %[thr]\n\t"       \
        "s_mov_b64 s[90:91], exec\n\t"                     \
        "v_fma_f64 %[t], " ACC ", %[cx], %[sacc]\n\t"      \
        "v_cmpx_le_f64_e32 vcc, %[slo], %[t]\n\t"          \
        "v_min_u32_e32 %[m], " KEY ", %[m]\n\t"            \
        "s_mov_b64 exec, s[90:91]\n\t"
    asm volatile(
        "s_mov_b32 s88, %[begin]\n\t"
        "s_mov_b64 exec, %[alive]\n\t"
        "1:\n\t"
        "s_load_dwordx16 s[72:87], %[base], s88\n\t"
        "s_add_u32 s88, s88, 64\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        JSV_MIX_ENTRY("s72", "s73", "s[74:75]")
        "s_cbranch_execz 3f\n\t"
        JSV_MIX_ENTRY("s76", "s77", "s[78:79]")
        JSV_MIX_ENTRY("s80", "s81", "s[82:83]")
        JSV_MIX_ENTRY("s84", "s85", "s[86:87]")
        "s_cmp_lt_u32 s88, %[end]\n\t"
        "s_cbranch_scc1 1b\n\t"
        "3:\n\t"
        "s_mov_b32 %[pos], s88\n\t"
        "s_mov_b64 exec, %[full]\n\t"
        "s_nop 1"
        : [m] "+v"(m), [t] "=&v"(t), [pos] "=&s"(pos)
        : [base] "s"(U.quads), [begin] "s"(qlo * 64u), [end] "s"(qhi * 64u), [full] "s"(full),
          [alive] "s"(alive),
          [thr] "v"(thr), [cx] "v"(s.hin[0]), [sacc] "v"(s.sacc), [slo] "s"(U.slo_raw)
        : "vcc", "scc", "s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", "s80", "s81", "s82",
          "s83", "s84", "s85", "s86", "s87", "s88", "s90", "s91");
#undef JSV_MIX_ENTRY
#else
    (void)thr; (void)t; (void)qlo; (void)qhi; (void)full; (void)alive;
#endif
    visits += (pos - qlo * 64u) / 16u;      // the stream ends early: counted with and without bounds
    const uint32_t cand = __builtin_elementwise_add_sat(s.k32, m);   // stays 0xFFFFFFFF if none
    best32 = best32 < cand ? best32 : cand;
}

// Objective mode, 64-bit keys: every candidate gets its objective and the
// lexicographic (objective, key) maximum.
template <bool BOUNDS>
__device__ __forceinline__ void loop_x64_obj(const LaneState& s, const Uniforms& U, uint32_t lo, uint32_t hi,
                                             Best& best, uint32_t& visits)
{
    const uint32_t worst = umax(s.smax, s.nxt[0]);
    uint32_t thr = worst <= U.sloq ? U.sloq - s.nxt[0] : 0u;
    if constexpr (BOUNDS) {
        if ((s.key >> U.idx_bits) + U.min_x_cost > U.bound) thr = 0;
        if (__builtin_amdgcn_ballot_w64(thr >= U.min_x_lat) == 0) return;
    }
    if (BOUNDS || U.mix) visits += hi - lo;
    const double cx = s.hin[0];
    const Entry JSV_CONST* tx = U.tab[0];
    for (uint32_t d = lo; d < hi; ++d) {
        const uint32_t lat = tx[d].lat;
        const uint64_t k = s.key + tx[d].key;
        const double A = __builtin_fma(tx[d].acc, cx, s.sacc);
        const uint32_t cost = (uint32_t)(k >> U.idx_bits);
        const bool ok = (lat <= thr) & (A >= U.slo_raw) & (U.capacity == 0 || cost <= U.capacity);   // Eq. 3, 13, 8
        const double obj = __builtin_fma(-U.beta, (double)cost, U.alpha_n * A);
        if (ok && better(obj, k, best.obj, best.key)) { best.obj = obj; best.key = k; }
    }
}

// One quad of the innermost stream as sixteen dwords: a single 64-byte scalar load.
typedef uint32_t QuadWords __attribute__((ext_vector_type(16)));
__device__ __forceinline__ QuadWords load_quad(const Quad JSV_CONST* q, uint32_t j)
{
    return *(const QuadWords JSV_CONST*)(q + j);
}
__device__ __forceinline__ double words_f64(uint32_t lo, uint32_t hi)
{
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// What the enumeration kernel is instantiated for.
constexpr int MODE_COST = 0;      // cheapest feasible
constexpr int MODE_OBJ  = 1;      // largest objective (Eq. 14)
constexpr int MODE_MIX  = 2;      // cheapest feasible, options with their own accuracies (Eq. 9, 10)
constexpr int MODE_MIXOBJ = 3;    // largest objective over such options
constexpr bool is_obj(int mode) { return mode == MODE_OBJ || mode == MODE_MIXOBJ; }
constexpr bool is_mix(int mode) { return mode == MODE_MIX || mode == MODE_MIXOBJ; }

// Objective mode, 32-bit local keys.  All candidates of one variant of position 0
// (other digits fixed) share their accuracy, so the one with the best objective is
// the cheapest feasible one: per variant the same masked minimum as in cost mode,
// then one objective and one (objective, key) comparison for the variant's winner.
// A variant whose cheapest candidate exceeds S_avail has no candidate within it.
//
// The objective itself (a conversion, two fp64 operations, three compares, three selects) is
// evaluated only where it can matter.  A_obj <= 1, so a candidate of cost c scores at most
// alpha - beta*c: once a lane holds a candidate of objective o, nothing costlier than
// (alpha - o)/beta can replace it.  That limit, S_avail, and the cost of the lane's fixed
// positions give one threshold on the 32-bit local key (klim); a variant whose winner lies
// above it in every lane of the wave is skipped with one compare.  Every candidate's latency
// test and minimum, and every variant's accuracy test, are still issued.
struct TileBest {
    uint32_t k32; double obj;
    uint32_t visits;    // wave-uniform: entries of position 0 this wave went through in the tile
    uint32_t klim;      // objective mode: local keys above it (fixed in-lane positions included) cannot matter
    uint32_t bound;     // wave-uniform: the cost bound as the wave knows it when the tile ends,
    double obj_seen;    // and (objective mode) the best objective of the instance it knows of
};

// With bounds, the cost bound moves while a tile runs.  At the points where a loop calls
// bound_take_in (before a digit or a run of the outermost in-lane position) the wave takes in what
// the instance's bound has become - the load issued at the previous such point, so nobody waits
// for it - and fetches it anew; where it calls bound_publish (after that digit or run), a wave one
// of whose lanes has found something better than the wave knew of lowers the bound for its own
// next steps and for every block working on the instance.  A stale value only excludes less;
// candidates as cheap as the bound stay in.  Cost modes: the bound is the cost of the cheapest
// candidate found that meets both SLOs.  Objective modes (Eq. 14): A_obj <= 1, so with an
// objective o reached nothing costlier than (alpha - o)/beta can match it (one unit of slack
// keeps the test clear of rounding and of equal objectives); single tuples also share o itself.
struct Moving {
    uint32_t fetched;                   // the bound, load in flight
    unsigned long long fetched_obj;     // the best objective, load in flight (objective mode, single tuples)
    double told;                        // per lane: the tile's best objective when the wave last published
};

template <int MODE>
__device__ __forceinline__ Moving bound_start(const Uniforms& V, const TileBest& tb)
{
    Moving mv;
    mv.fetched = V.bound;
    mv.fetched_obj = ordered_bits(-__builtin_inf());
    mv.told = tb.obj;
    return mv;
}

template <int MODE>
__device__ __forceinline__ void bound_take_in(Uniforms& V, Moving& mv)
{
    const uint32_t seen = (uint32_t)__builtin_amdgcn_readfirstlane((int)mv.fetched);
    V.bound = seen < V.bound ? seen : V.bound;
    mv.fetched = __hip_atomic_load(V.bound_at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if constexpr (MODE == MODE_OBJ) {
        const double oo = from_ordered_bits(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(mv.fetched_obj >> 32)) << 32) |
                                            (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)mv.fetched_obj));
        V.obj_seen = oo > V.obj_seen ? oo : V.obj_seen;
        mv.fetched_obj = __hip_atomic_load(V.best_obj_at, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int MODE>
__device__ __forceinline__ void bound_publish(const LaneState& s, Uniforms& V, const TileBest& tb, Moving& mv)
{
    if constexpr (!is_obj(MODE)) {
        // (the tile's best local key so far -> the total cost of that candidate)
        const uint32_t c = tb.k32 != 0xFFFFFFFFu ? s.cost_out + (tb.k32 >> V.lb) : 0xFFFFFFFFu;
        if (__builtin_amdgcn_ballot_w64(c < V.bound) == 0) return;
        const uint32_t wc = (uint32_t)wave_min((uint64_t)c);
        V.bound = wc;
        if ((threadIdx.x & 63u) == 0) atomicMin(V.bound_at, wc);
    } else {
        if (__builtin_amdgcn_ballot_w64(tb.obj > mv.told) == 0) return;
        mv.told = tb.obj;
        const unsigned long long ob = ~wave_min(~ordered_bits(tb.obj));     // the largest of the lanes' objectives
        const double o = from_ordered_bits(ob);
        if constexpr (MODE == MODE_OBJ) {
            if (o > V.obj_seen) {
                V.obj_seen = o;
                if ((threadIdx.x & 63u) == 0) atomicMax(V.best_obj_at, ob);
            }
        }
        if (V.beta > 1e-9 * (V.alpha + 1.0)) {      // else rounding could reach a unit of cost
            const double lim = (V.alpha - o) / V.beta;
            if (lim >= 0.0 && lim < 2147483000.0) {
                const uint32_t wc = (uint32_t)lim + 1u;
                if (wc < V.bound) {
                    V.bound = wc;
                    if ((threadIdx.x & 63u) == 0) atomicMin(V.bound_at, wc);
                }
            }
        }
    }
}

// Largest local key that can still matter for a lane whose positions outside the lane loops cost
// `cost_out` and that already holds a candidate of objective `have` (-inf: none).  0: none can
// (real keys are at least 1 << lb: every task costs at least one unit).
// `top`: what alpha * A_obj can be at most among the candidates in question - alpha itself
// (A_obj <= 1), or less where their accuracy is known to stay below some value.
__device__ __forceinline__ uint32_t key_limit(const Uniforms& U, uint32_t cost_out, double have, double top)
{
    // Eq. 8, and what any block has made of the instance's shared limit so far (at most S_avail)
    uint32_t cost_lim = U.bound;
    have = have > U.obj_seen ? have : U.obj_seen;           // (-inf where no objective is shared)
    if (U.inv_beta > 0.0 && have > -__builtin_inf()) {
        const double lim = (top - have) * U.inv_beta;
        // one unit of slack keeps rounding and equal objectives out of the decision
        if (lim < 4294967000.0) { const uint32_t l = (lim > 0.0 ? (uint32_t)lim : 0u) + 1u; cost_lim = l < cost_lim ? l : cost_lim; }
    }
    if (cost_lim < cost_out) return 0u;
    const uint64_t k = (((uint64_t)(cost_lim - cost_out) + 1u) << U.lb) - 1u;
    return k > 0xFFFFFFFEull ? 0xFFFFFFFEu : (uint32_t)k;
}

// m: the variant's cheapest local key among the candidates that pass Eq. 3 (0xFFFFFFFF: none),
// t: its A_raw, mlim: klim less the fixed in-lane positions' key.
__device__ __forceinline__ void fold_variant(const LaneState& s, const Uniforms& U, uint32_t m, double t, TileBest& tb,
                                             uint32_t& mlim)
{
    const bool hit = m <= mlim;                                  // (mlim < 0xFFFFFFFF)
    const uint32_t k = s.k32 + m;
    const uint32_t cost = s.cost_out + (k >> U.lb);
    const double obj = __builtin_fma(-U.beta, (double)cost, U.alpha_n * t);
    const bool improved = hit && (obj > tb.obj || (obj == tb.obj && k < tb.k32));
    if (improved) { tb.obj = obj; tb.k32 = k; }
    if (__builtin_amdgcn_ballot_w64(improved) != 0) {            // rare once a lane holds something good
        const uint32_t kl = key_limit(U, s.cost_out, tb.obj, U.alpha);
        tb.klim = kl < tb.klim ? kl : tb.klim;
        mlim = __builtin_elementwise_sub_sat(tb.klim, s.k32);
    }
}

template <bool BOUNDS>
__device__ __forceinline__ void loop_x32_obj(const LaneState& s, const Uniforms& U, uint32_t qlo, uint32_t qhi,
                                             uint64_t full, TileBest& tb)
{
    const uint32_t thr = __builtin_elementwise_sub_sat(U.sloq, s.nxt[0]);
    uint64_t alive;
    if constexpr (BOUNDS) {
        // also out: lanes whose fixed positions plus the cheapest entry here cost more than the bound
        const uint32_t fixed = s.cost_out + (s.k32 >> U.lb);
        alive = __builtin_amdgcn_ballot_w64((s.smax <= U.sloq) & (thr >= U.min_x_lat) & (fixed + U.min_x_cost <= U.bound));
    } else alive = __builtin_amdgcn_ballot_w64(s.smax <= U.sloq);
    if (BOUNDS && alive == 0) return;
    if constexpr (BOUNDS) tb.visits += (qhi - qlo) * 4u;
    const Quad JSV_CONST* q = U.quads;
    uint32_t m = 0xFFFFFFFFu;
    uint32_t mlim = __builtin_elementwise_sub_sat(tb.klim, s.k32);
    double t = 0.0;
    uint64_t ok = 0;
    // every quad comes in through one 64-byte scalar load, issued one quad ahead of its use
    QuadWords w = load_quad(q, qlo);
    for (uint32_t j = qlo; j < qhi; ++j) {
        const QuadWords cur = w;
        w = load_quad(q, j + 1 < qhi ? j + 1 : j);
        if (cur[10] != 0) {                                     // a new variant (or the tile's range) starts
            if (__builtin_amdgcn_ballot_w64(m <= mlim) != 0) fold_variant(s, U, m, t, tb, mlim);   // some lane's winner can matter
            t = __builtin_fma(words_f64(cur[8], cur[9]), s.hin[0], s.sacc);
            ok = alive & __builtin_amdgcn_ballot_w64(t >= U.slo_raw);
            m = 0xFFFFFFFFu;
        }
#if defined(__HIP_DEVICE_COMPILE__)
        // the quad's candidates in ascending latency under the variant's mask (see loop_x32)
        asm volatile(
            "s_mov_b64 exec, %[ok]\n\t"
            "v_cmpx_le_u32_e32 vcc, %[l0], %[thr]\n\t"
            "v_min_u32_e32 %[m], %[k0], %[m]\n\t"
            "v_cmpx_le_u32_e32 vcc, %[l1], %[thr]\n\t"
            "v_min_u32_e32 %[m], %[k1], %[m]\n\t"
            "v_cmpx_le_u32_e32 vcc, %[l2], %[thr]\n\t"
            "v_min_u32_e32 %[m], %[k2], %[m]\n\t"
            "v_cmpx_le_u32_e32 vcc, %[l3], %[thr]\n\t"
            "v_min_u32_e32 %[m], %[k3], %[m]\n\t"
            "s_mov_b64 exec, %[full]\n\t"
            "s_nop 1"
            : [m] "+v"(m)
            : [ok] "s"(ok), [full] "s"(full), [thr] "v"(thr),
              [l0] "s"(cur[0]), [k0] "s"(cur[1]), [l1] "s"(cur[2]), [k1] "s"(cur[3]),
              [l2] "s"(cur[4]), [k2] "s"(cur[5]), [l3] "s"(cur[6]), [k3] "s"(cur[7])
            : "vcc");
#else
        (void)thr; (void)full; (void)ok;
#endif
    }
    if (__builtin_amdgcn_ballot_w64(m <= mlim) != 0) fold_variant(s, U, m, t, tb, mlim);
}

// Objective mode over mixtures, 32-bit local keys.  Every entry has its own accuracy and so
// its own objective; the stream is in ascending latency (QuadM).  Per candidate: the latency
// compare (once no lane of the wave passes it, nothing later can: the loop ends), the
// accuracy fma and compare, and one compare of the entry's key against the lane's limit
// (see key_limit); the objective is evaluated only where all three pass in some lane.
template <bool BOUNDS>
__device__ __forceinline__ void loop_x32_mixobj(const LaneState& s, const Uniforms& U, uint32_t qlo, uint32_t qhi, TileBest& tb)
{
    const uint32_t thr = __builtin_elementwise_sub_sat(U.sloq, s.nxt[0]);
    bool lane_ok = s.smax <= U.sloq;
    if constexpr (BOUNDS) {
        const uint32_t fixed = s.cost_out + (s.k32 >> U.lb);
        lane_ok = lane_ok & (thr >= U.min_x_lat) & (fixed + U.min_x_cost <= U.bound);
        if (__builtin_amdgcn_ballot_w64(lane_ok) == 0) return;
    }
    uint32_t mlim = __builtin_elementwise_sub_sat(tb.klim, s.k32);
    const Quad JSV_CONST* q = U.quads;                       // (QuadM records: four entries of lat, key, accuracy)
    uint32_t seen = 0;
    QuadWords w = load_quad(q, qlo);
    for (uint32_t j = qlo; j < qhi; ++j) {
        const QuadWords cur = w;                                // one 64-byte scalar load per quad, one quad ahead
        w = load_quad(q, j + 1 < qhi ? j + 1 : j);
        bool done = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t lat = cur[4 * e], key = cur[4 * e + 1];
            const bool fast = lane_ok & (lat <= thr);                             // Eq. 3
            if (__builtin_amdgcn_ballot_w64(fast) == 0) { done = true; break; }   // (padding entries end here too)
            ++seen;
            const double t = __builtin_fma(words_f64(cur[4 * e + 2], cur[4 * e + 3]), s.hin[0], s.sacc);
            const bool cand = fast & (t >= U.slo_raw) & (key <= mlim);            // Eq. 13; can it matter?
            if (__builtin_amdgcn_ballot_w64(cand) != 0) {
                const uint32_t k = s.k32 + key;
                const uint32_t cost = s.cost_out + (k >> U.lb);
                const double obj = __builtin_fma(-U.beta, (double)cost, U.alpha_n * t);
                const bool improved = cand && (obj > tb.obj || (obj == tb.obj && k < tb.k32));
                if (improved) { tb.obj = obj; tb.k32 = k; }
                if (__builtin_amdgcn_ballot_w64(improved) != 0) {
                    const uint32_t kl = key_limit(U, s.cost_out, tb.obj, U.alpha);
                    tb.klim = kl < tb.klim ? kl : tb.klim;
                    mlim = __builtin_elementwise_sub_sat(tb.klim, s.k32);
                }
            }
        }
        if (done) break;
    }
    if constexpr (BOUNDS) tb.visits += seen;
}

template <bool W32, int MODE, bool BOUNDS>
__device__ __forceinline__ void loop_x(const LaneState& s, const Uniforms& U, uint32_t lo, uint32_t hi,
                                       uint64_t full, Best& best, TileBest& tb)
{
    if constexpr (is_obj(MODE)) {
        if constexpr (W32) {
            // Two passes.  The first is the cost modes' loop: the cheapest candidate of this pass
            // that meets Eq. 3 and 13, over all variants, at two vector instructions per candidate.
            // Only if that one lies within the lane's key limit in some lane of the wave can the
            // pass hold a new best objective (see key_limit); then the second pass goes through it
            // again variant by variant (mixtures: entry by entry) and evaluates objectives.
            uint32_t cheapest = 0xFFFFFFFFu, unused = 0;
            if constexpr (is_mix(MODE)) loop_x32_mix<BOUNDS>(s, U, lo, hi, full, cheapest, tb.visits);
            else loop_x32<BOUNDS>(s, U, lo, hi, full, cheapest, tb.visits);
            bool want = cheapest <= tb.klim;
            if constexpr (is_mix(MODE)) {
                if (__builtin_amdgcn_ballot_w64(want) != 0) {
                    // Exactly: no option of position 0 is more accurate than its most accurate one and
                    // none that passes costs less than the cheapest, so nothing in this pass scores more
                    // than this (same operations as the objective itself, which are monotone).
                    const double top = U.alpha_n * __builtin_fma(U.xacc[0], s.hin[0], s.sacc);
                    const uint32_t cost = s.cost_out + (cheapest >> U.lb);
                    want = want & (__builtin_fma(-U.beta, (double)cost, top) >= tb.obj);
                }
            }
            if (__builtin_amdgcn_ballot_w64(want) != 0) {
                TileBest again = tb;
                again.visits = 0;
                if constexpr (is_mix(MODE)) loop_x32_mixobj<BOUNDS>(s, U, lo, hi, again);
                else loop_x32_obj<BOUNDS>(s, U, lo, hi, full, again);
                tb.k32 = again.k32; tb.obj = again.obj; tb.klim = again.klim;
            }
            (void)unused;
        } else loop_x64_obj<BOUNDS>(s, U, lo, hi, best, tb.visits);
    } else if constexpr (MODE == MODE_MIX) {
        if constexpr (W32) loop_x32_mix<BOUNDS>(s, U, lo, hi, full, tb.k32, tb.visits);
        else loop_x64<BOUNDS>(s, U, lo, hi, best.key, tb.visits);
    } else {
        if constexpr (W32) loop_x32<BOUNDS>(s, U, lo, hi, full, tb.k32, tb.visits);
        else loop_x64<BOUNDS>(s, U, lo, hi, best.key, tb.visits);
    }
}

// Positions 1 and 0 together, single tuples, 32-bit keys, at most MAX_XVAR variants in position
// 0's stream.  The accuracy of a candidate (Eq. 11-13) depends on the variants only, so while
// position 1 stays with one accuracy the outcome of Eq. 13 for each variant of position 0 is
// the same: it is evaluated once per variant pair - the same fma and compare as in loop_x32 -
// and kept as one execution mask per variant of position 0 in scalar registers.  Along the
// digits of position 1 only latencies and keys change, and G of them (slots) go through
// position 0's stream together: every record that is loaded serves G digits, each with its own
// latency threshold, set of live lanes and running minimum.
//
// The stream is walked in its QuadC copy, variant by variant, in code written out per place of
// the variant in the stream: per slot and record one scalar AND puts the variant's mask and
// the slot's live lanes into EXEC, then per candidate the two vector instructions of loop_x32
// follow (a lane that fails one candidate's latency test sits out the rest of the record).
// Records alternate between two register sets (A: s[72:79], B: s[80:87]); the next record's
// load is issued before the current one's vector instructions and waited for after them.  s88
// is the byte offset of the next record to load, so the record in flight lies 32 bytes before
// it: it still belongs to variant v while s88 <= xqe[v], and the stream is done once s88 > its
// length (the record then in flight is the spare one behind the stream).  A variant may end in
// either register set, hence two ways into every block: labels 10(v+1)+1 and +3 (start of
// variant v with the current record in A, in B), +2 and +4 (the loop itself), 99 the end.
//
// SKIP (with bounds on): a slot none of whose lanes can take the record's fastest candidate
// leaves the record at once.
#define JSV_SLOT(L0, K0, L1, K1, L2, K2, L3, K3, MASK, ALIVE, THR, M, SKIP)                        \
        "s_and_b64 exec, " MASK ", " ALIVE "\n\t"                                                  \
        "v_cmpx_le_u32_e32 vcc, " L0 ", " THR "\n\t"                                               \
        SKIP                                                                                       \
        "v_min_u32_e32 " M ", " K0 ", " M "\n\t"                                                   \
        "v_cmpx_le_u32_e32 vcc, " L1 ", " THR "\n\t"                                               \
        "v_min_u32_e32 " M ", " K1 ", " M "\n\t"                                                   \
        "v_cmpx_le_u32_e32 vcc, " L2 ", " THR "\n\t"                                               \
        "v_min_u32_e32 " M ", " K2 ", " M "\n\t"                                                   \
        "v_cmpx_le_u32_e32 vcc, " L3 ", " THR "\n\t"                                               \
        "v_min_u32_e32 " M ", " K3 ", " M "\n\t"                                                   \
        "5:\n\t"
#define JSV_SLOTS_A1(MASK, SKIP) JSV_SLOT("s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", MASK, "%[a0]", "%[t0]", "%[r0]", SKIP)
#define JSV_SLOTS_B1(MASK, SKIP) JSV_SLOT("s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", MASK, "%[a0]", "%[t0]", "%[r0]", SKIP)
#define JSV_SLOTS_A2(MASK, SKIP) JSV_SLOTS_A1(MASK, SKIP) JSV_SLOT("s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", MASK, "%[a1]", "%[t1]", "%[r1]", SKIP)
#define JSV_SLOTS_B2(MASK, SKIP) JSV_SLOTS_B1(MASK, SKIP) JSV_SLOT("s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", MASK, "%[a1]", "%[t1]", "%[r1]", SKIP)
#define JSV_SLOTS_A3(MASK, SKIP) JSV_SLOTS_A2(MASK, SKIP)                                          \
        JSV_SLOT("s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", MASK, "%[a2]", "%[t2]", "%[r2]", SKIP)
#define JSV_SLOTS_B3(MASK, SKIP) JSV_SLOTS_B2(MASK, SKIP)                                          \
        JSV_SLOT("s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", MASK, "%[a2]", "%[t2]", "%[r2]", SKIP)
#define JSV_SLOTS_A4(MASK, SKIP) JSV_SLOTS_A3(MASK, SKIP)                                          \
        JSV_SLOT("s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", MASK, "%[a3]", "%[t3]", "%[r3]", SKIP)
#define JSV_SLOTS_B4(MASK, SKIP) JSV_SLOTS_B3(MASK, SKIP)                                          \
        JSV_SLOT("s80", "s81", "s82", "s83", "s84", "s85", "s86", "s87", MASK, "%[a3]", "%[t3]", "%[r3]", SKIP)
#define JSV_XV_HALF(START, LOOP, SLOTS, NEXTREGS, STAY, LEAVE, QE)                                 \
        START ":\n\t"                                                                              \
        "s_cmp_gt_u32 s88, %[endb]\n\t"                                                            \
        "s_cbranch_scc1 99f\n\t"                                                                   \
        LOOP ":\n\t"                                                                               \
        "s_load_dwordx8 " NEXTREGS ", %[base], s88\n\t"                                            \
        "s_add_u32 s88, s88, 32\n\t"                                                               \
        SLOTS                                                                                      \
        "s_waitcnt lgkmcnt(0)\n\t"                                                                 \
        "s_cmp_le_u32 s88, " QE "\n\t"                                                             \
        "s_cbranch_scc1 " STAY "\n\t"                                                              \
        "s_branch " LEAVE "\n\t"
// variant block N (labels N1..N4), ways out to the next block: XA (current record in A), XB (in B)
#define JSV_XV(G, N, XA, XB, MASK, QE, SKIP)                                                       \
        JSV_XV_HALF(N "1", N "2", JSV_SLOTS_A##G(MASK, SKIP), "s[80:87]", N "4f", XB, QE)          \
        JSV_XV_HALF(N "3", N "4", JSV_SLOTS_B##G(MASK, SKIP), "s[72:79]", N "2b", XA, QE)
#define JSV_XV_ALL(G, SKIP)                                                                        \
        "s_mov_b32 s88, 0\n\t"                                                                     \
        "s_load_dwordx8 s[72:79], %[base], s88\n\t"                                                \
        "s_mov_b32 s88, 32\n\t"                                                                    \
        "s_waitcnt lgkmcnt(0)\n\t"                                                                 \
        JSV_XV(G, "1", "21f", "23f", "%[m0]", "%[q0]", SKIP) JSV_XV(G, "2", "31f", "33f", "%[m1]", "%[q1]", SKIP) \
        JSV_XV(G, "3", "41f", "43f", "%[m2]", "%[q2]", SKIP) JSV_XV(G, "4", "51f", "53f", "%[m3]", "%[q3]", SKIP) \
        JSV_XV(G, "5", "61f", "63f", "%[m4]", "%[q4]", SKIP) JSV_XV(G, "6", "71f", "73f", "%[m5]", "%[q5]", SKIP) \
        JSV_XV(G, "7", "81f", "83f", "%[m6]", "%[q6]", SKIP) JSV_XV(G, "8", "99f", "99f", "%[m7]", "%[q7]", SKIP) \
        "99:\n\t"                                                                                  \
        "s_mov_b64 exec, %[full]\n\t"                                                              \
        "s_nop 1"
#define JSV_XV_COMMON_IN                                                                           \
          [base] "s"(base), [endb] "s"(endb), [full] "s"(full),                                    \
          [m0] "s"(mk[0]), [m1] "s"(mk[1]), [m2] "s"(mk[2]), [m3] "s"(mk[3]),                      \
          [m4] "s"(mk[4]), [m5] "s"(mk[5]), [m6] "s"(mk[6]), [m7] "s"(mk[7]),                      \
          [q0] "s"(qe[0]), [q1] "s"(qe[1]), [q2] "s"(qe[2]), [q3] "s"(qe[3]),                      \
          [q4] "s"(qe[4]), [q5] "s"(qe[5]), [q6] "s"(qe[6]), [q7] "s"(qe[7])
#define JSV_XV_CLOBBER                                                                             \
          "vcc", "scc", "s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", "s80", "s81", "s82", \
          "s83", "s84", "s85", "s86", "s87", "s88"

// G = 4, 3, 2 or 1 slots: thresholds thr[g], live lanes go[g], running minima m[g] (in and out).
// base: the stream's records (position 0's QuadC copy, or one digit's block of the pair stream).
template <int G, bool BOUNDS>
__device__ __forceinline__ void loop_x32_masked(const QuadC JSV_CONST* base, const uint32_t (&thr)[4], const uint64_t (&go)[4],
                                                const uint64_t (&mk)[MAX_XVAR], const uint32_t (&qe)[MAX_XVAR],
                                                uint32_t endb, uint64_t full, uint32_t (&m)[4])
{
    static_assert(MAX_XVAR == 8, "the blocks above are written out for eight variants");
    static_assert(G >= 1 && G <= 4, "slots");
#if defined(__HIP_DEVICE_COMPILE__)
    if constexpr (G == 4) {
        if constexpr (BOUNDS)
            asm volatile(JSV_XV_ALL(4, "s_cbranch_execz 5f\n\t")
                : [r0] "+v"(m[0]), [r1] "+v"(m[1]), [r2] "+v"(m[2]), [r3] "+v"(m[3])
                : JSV_XV_COMMON_IN, [t0] "v"(thr[0]), [t1] "v"(thr[1]), [t2] "v"(thr[2]), [t3] "v"(thr[3]),
                  [a0] "s"(go[0]), [a1] "s"(go[1]), [a2] "s"(go[2]), [a3] "s"(go[3])
                : JSV_XV_CLOBBER);
        else
            asm volatile(JSV_XV_ALL(4, "")
                : [r0] "+v"(m[0]), [r1] "+v"(m[1]), [r2] "+v"(m[2]), [r3] "+v"(m[3])
                : JSV_XV_COMMON_IN, [t0] "v"(thr[0]), [t1] "v"(thr[1]), [t2] "v"(thr[2]), [t3] "v"(thr[3]),
                  [a0] "s"(go[0]), [a1] "s"(go[1]), [a2] "s"(go[2]), [a3] "s"(go[3])
                : JSV_XV_CLOBBER);
    } else if constexpr (G == 3) {
        if constexpr (BOUNDS)
            asm volatile(JSV_XV_ALL(3, "s_cbranch_execz 5f\n\t")
                : [r0] "+v"(m[0]), [r1] "+v"(m[1]), [r2] "+v"(m[2])
                : JSV_XV_COMMON_IN, [t0] "v"(thr[0]), [t1] "v"(thr[1]), [t2] "v"(thr[2]),
                  [a0] "s"(go[0]), [a1] "s"(go[1]), [a2] "s"(go[2])
                : JSV_XV_CLOBBER);
        else
            asm volatile(JSV_XV_ALL(3, "")
                : [r0] "+v"(m[0]), [r1] "+v"(m[1]), [r2] "+v"(m[2])
                : JSV_XV_COMMON_IN, [t0] "v"(thr[0]), [t1] "v"(thr[1]), [t2] "v"(thr[2]),
                  [a0] "s"(go[0]), [a1] "s"(go[1]), [a2] "s"(go[2])
                : JSV_XV_CLOBBER);
    } else if constexpr (G == 2) {
        if constexpr (BOUNDS)
            asm volatile(JSV_XV_ALL(2, "s_cbranch_execz 5f\n\t")
                : [r0] "+v"(m[0]), [r1] "+v"(m[1])
                : JSV_XV_COMMON_IN, [t0] "v"(thr[0]), [t1] "v"(thr[1]), [a0] "s"(go[0]), [a1] "s"(go[1])
                : JSV_XV_CLOBBER);
        else
            asm volatile(JSV_XV_ALL(2, "")
                : [r0] "+v"(m[0]), [r1] "+v"(m[1])
                : JSV_XV_COMMON_IN, [t0] "v"(thr[0]), [t1] "v"(thr[1]), [a0] "s"(go[0]), [a1] "s"(go[1])
                : JSV_XV_CLOBBER);
    } else {
        if constexpr (BOUNDS)
            asm volatile(JSV_XV_ALL(1, "s_cbranch_execz 5f\n\t")
                : [r0] "+v"(m[0]) : JSV_XV_COMMON_IN, [t0] "v"(thr[0]), [a0] "s"(go[0]) : JSV_XV_CLOBBER);
        else
            asm volatile(JSV_XV_ALL(1, "")
                : [r0] "+v"(m[0]) : JSV_XV_COMMON_IN, [t0] "v"(thr[0]), [a0] "s"(go[0]) : JSV_XV_CLOBBER);
    }
#else
    (void)base; (void)thr; (void)go; (void)mk; (void)qe; (void)endb; (void)full; (void)m;
#endif
}
#undef JSV_XV_CLOBBER
#undef JSV_XV_COMMON_IN
#undef JSV_XV_ALL
#undef JSV_XV
#undef JSV_XV_HALF
#undef JSV_SLOTS_B4
#undef JSV_SLOTS_A4
#undef JSV_SLOTS_B3
#undef JSV_SLOTS_A3
#undef JSV_SLOTS_B2
#undef JSV_SLOTS_A2
#undef JSV_SLOTS_B1
#undef JSV_SLOTS_A1
#undef JSV_SLOT

// Eq. 13 for every variant of position 0, given what the other positions contribute to A_raw:
// mk[v] = lanes with fma(xacc[v], hin0, sacc) >= slo_raw, v < nvx; the others 0.  One
// 64-byte scalar load brings all MAX_XVAR accuracies.
__device__ __forceinline__ void variant_masks(const Uniforms& U, uint32_t nvx, double hin0, double sacc,
                                              uint64_t (&mk)[MAX_XVAR])
{
    static_assert(MAX_XVAR == 8, "written out for eight variants");
#if defined(__HIP_DEVICE_COMPILE__)
    double t;
#define JSV_VM(N, REGS, OUT)                                                                       \
        "s_cmp_lt_u32 %[nvx], " N "\n\t"                                                           \
        "s_cbranch_scc1 1f\n\t"                                                                    \
        "v_fma_f64 %[t], " REGS ", %[hin0], %[sacc]\n\t"                                           \
        "v_cmp_le_f64_e64 " OUT ", %[slo], %[t]\n\t"
    asm volatile(
        "s_load_dwordx16 s[72:87], %[xacc], 0x0\n\t"
        "s_mov_b64 %[m1], 0\n\t"
        "s_mov_b64 %[m2], 0\n\t"
        "s_mov_b64 %[m3], 0\n\t"
        "s_mov_b64 %[m4], 0\n\t"
        "s_mov_b64 %[m5], 0\n\t"
        "s_mov_b64 %[m6], 0\n\t"
        "s_mov_b64 %[m7], 0\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fma_f64 %[t], s[72:73], %[hin0], %[sacc]\n\t"
        "v_cmp_le_f64_e64 %[m0], %[slo], %[t]\n\t"
        JSV_VM("2", "s[74:75]", "%[m1]") JSV_VM("3", "s[76:77]", "%[m2]") JSV_VM("4", "s[78:79]", "%[m3]")
        JSV_VM("5", "s[80:81]", "%[m4]") JSV_VM("6", "s[82:83]", "%[m5]") JSV_VM("7", "s[84:85]", "%[m6]")
        JSV_VM("8", "s[86:87]", "%[m7]")
        "1:"
        : [m0] "=&s"(mk[0]), [m1] "=&s"(mk[1]), [m2] "=&s"(mk[2]), [m3] "=&s"(mk[3]),
          [m4] "=&s"(mk[4]), [m5] "=&s"(mk[5]), [m6] "=&s"(mk[6]), [m7] "=&s"(mk[7]), [t] "=&v"(t)
        : [xacc] "s"(U.xacc), [nvx] "s"(nvx), [hin0] "v"(hin0), [sacc] "v"(sacc), [slo] "s"(U.slo_raw)
        : "scc", "s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", "s80", "s81", "s82",
          "s83", "s84", "s85", "s86", "s87");
#undef JSV_VM
#else
    (void)U; (void)nvx; (void)hin0; (void)sacc; (void)mk;
#endif
}

// The same, and the largest A_raw among the variants of position 0 (objective mode: no candidate
// of this combination of variants of the other positions can be more accurate).
__device__ __forceinline__ void variant_masks_tmax(const Uniforms& U, uint32_t nvx, double hin0, double sacc,
                                                   uint64_t (&mk)[MAX_XVAR], double& tmax)
{
    static_assert(MAX_XVAR == 8, "written out for eight variants");
#if defined(__HIP_DEVICE_COMPILE__)
    double t, tm;
#define JSV_VM(N, REGS, OUT)                                                                       \
        "s_cmp_lt_u32 %[nvx], " N "\n\t"                                                           \
        "s_cbranch_scc1 1f\n\t"                                                                    \
        "v_fma_f64 %[t], " REGS ", %[hin0], %[sacc]\n\t"                                           \
        "v_cmp_le_f64_e64 " OUT ", %[slo], %[t]\n\t"                                               \
        "v_max_f64 %[tm], %[tm], %[t]\n\t"
    asm volatile(
        "s_load_dwordx16 s[72:87], %[xacc], 0x0\n\t"
        "s_mov_b64 %[m1], 0\n\t"
        "s_mov_b64 %[m2], 0\n\t"
        "s_mov_b64 %[m3], 0\n\t"
        "s_mov_b64 %[m4], 0\n\t"
        "s_mov_b64 %[m5], 0\n\t"
        "s_mov_b64 %[m6], 0\n\t"
        "s_mov_b64 %[m7], 0\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fma_f64 %[tm], s[72:73], %[hin0], %[sacc]\n\t"
        "v_cmp_le_f64_e64 %[m0], %[slo], %[tm]\n\t"
        JSV_VM("2", "s[74:75]", "%[m1]") JSV_VM("3", "s[76:77]", "%[m2]") JSV_VM("4", "s[78:79]", "%[m3]")
        JSV_VM("5", "s[80:81]", "%[m4]") JSV_VM("6", "s[82:83]", "%[m5]") JSV_VM("7", "s[84:85]", "%[m6]")
        JSV_VM("8", "s[86:87]", "%[m7]")
        "1:"
        : [m0] "=&s"(mk[0]), [m1] "=&s"(mk[1]), [m2] "=&s"(mk[2]), [m3] "=&s"(mk[3]),
          [m4] "=&s"(mk[4]), [m5] "=&s"(mk[5]), [m6] "=&s"(mk[6]), [m7] "=&s"(mk[7]), [t] "=&v"(t), [tm] "=&v"(tm)
        : [xacc] "s"(U.xacc), [nvx] "s"(nvx), [hin0] "v"(hin0), [sacc] "v"(sacc), [slo] "s"(U.slo_raw)
        : "scc", "s72", "s73", "s74", "s75", "s76", "s77", "s78", "s79", "s80", "s81", "s82",
          "s83", "s84", "s85", "s86", "s87");
#undef JSV_VM
    tmax = tm;
#else
    (void)U; (void)nvx; (void)hin0; (void)sacc; (void)mk; tmax = 0.0;
#endif
}

// Objective mode: what can still matter among the candidates whose A_raw is at most tmax (one
// combination of variants of positions 1 and 2, any variant of position 0): the key limit with
// alpha_n * tmax in place of alpha, never above tb.klim, and the same as a total cost.
__device__ __forceinline__ void combination_limits(const Uniforms& U, const TileBest& tb, uint32_t cost_out, double an_tmax,
                                                   uint32_t& klim_blk, uint32_t& clim_abs)
{
    const uint32_t k = key_limit(U, cost_out, tb.obj, an_tmax);
    klim_blk = k < tb.klim ? k : tb.klim;
    // ((c - cost_out + 1) << lb) - 1 back to c; a limit too large for a key stands for "none"
    clim_abs = klim_blk == 0u ? 0u
             : klim_blk == 0xFFFFFFFEu ? 0xFFFFFFFFu
             : __builtin_elementwise_add_sat(((klim_blk + 1u) >> U.lb) - 1u, cost_out);
}

typedef uint32_t YWords __attribute__((ext_vector_type(4), aligned(4)));       // four digits' latencies or keys

// The digits [d, re) of one run of position 1, four at a time, against position 0's stream.
// What the positions fixed so far give: smax (latest source so far), thr0 = sloq -sat nxt[0],
// room1 = sloq -sat nxt[1], alive0 = lanes with smax <= sloq, k32 and cost_out.  mk: the
// accuracy outcome per variant of position 0 for this run.  make_s1(digit): the full lane
// state with that digit of position 1 fixed (objective mode's second pass only).
template <int MODE, bool BOUNDS, bool E01, typename MakeS1>
__device__ __forceinline__ void y_batches(const Uniforms& U, uint32_t smax, uint32_t thr0, uint32_t room1, uint64_t alive0,
                                          uint32_t k32, uint32_t cost_out, uint32_t d, uint32_t re,
                                          const uint64_t (&mk)[MAX_XVAR], const uint32_t (&qe)[MAX_XVAR], uint32_t endb,
                                          uint32_t x_hi, uint64_t full, TileBest& tb, MakeS1 make_s1,
                                          uint32_t klim_blk = 0xFFFFFFFEu, uint32_t clim_abs = 0xFFFFFFFFu, double an_tmax = 0.0)
{
    // Position 1 is either a successor of position 0 (its only possible predecessor; E01) or a
    // source: in the first case its tail changes position 0's latency threshold, in the second
    // the lanes that still meet the latency SLO.
    constexpr uint32_t e01 = E01 ? 1u : 0u;
    constexpr uint32_t src1 = E01 ? 0u : 1u;
    if constexpr (BOUNDS) {
        // The digits from d to the end of their run as a whole first: with the cheapest and the fastest
        // of them, can any lane stay within the cost bound and leave position 0 a candidate?
        const uint32_t rk = U.yrk[d], rl = U.yrl[d];
        const uint32_t most = E01 ? umin(thr0, __builtin_elementwise_sub_sat(room1, rl)) : thr0;
        const uint32_t fixed = cost_out + ((k32 + rk) >> U.lb);
        const uint32_t within = MODE == MODE_OBJ ? umin(clim_abs, U.bound) : U.bound;
        bool can = (smax <= U.sloq) & (most >= U.min_x_lat) & (fixed + U.min_x_cost <= within);
        if constexpr (!E01) can = can & (rl <= room1);
        if (__builtin_amdgcn_ballot_w64(can) == 0) return;
    }
    uint32_t best_rel = 0xFFFFFFFFu;        // cost modes: the run's minimum of position 1's key plus position 0's
    for (; d < re; d += 4) {
        // four digits at a time, two 16-byte scalar loads
        const YWords lat4 = *(const YWords JSV_CONST*)(U.ylat + d);
        const YWords key4 = *(const YWords JSV_CONST*)(U.yk32 + d);
        const uint32_t n = re - d;
        uint32_t thr[4], m[4];
        uint64_t go[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            // With tail = lat + nxt[1] (the digit's latency to the sinks) and room1 = sloq -sat nxt[1]:
            // sloq -sat max(nxt[0], tail) = min(thr0, room1 -sat lat), and
            // max(smax, tail) <= sloq  <=>  smax <= sloq and lat <= room1 (latencies are >= 1).
            const uint32_t lat = lat4[g];
            bool meets = smax <= U.sloq;
            thr[g] = thr0; go[g] = alive0; m[g] = 0xFFFFFFFFu;
            if (e01 != 0) thr[g] = umin(thr0, __builtin_elementwise_sub_sat(room1, lat));
            if (src1 != 0) { meets = meets & (lat <= room1); go[g] = __builtin_amdgcn_ballot_w64(meets); }
            if constexpr (BOUNDS) {
                // also out: lanes whose fixed positions plus the cheapest entry of position 0 cost more than the bound
                const uint32_t fixed = cost_out + ((k32 + key4[g]) >> U.lb);
                // (objective mode: the bound of this combination of variants, see combination_limits)
                const uint32_t within = MODE == MODE_OBJ ? umin(clim_abs, U.bound) : U.bound;
                go[g] = __builtin_amdgcn_ballot_w64(meets & (thr[g] >= U.min_x_lat) & (fixed + U.min_x_cost <= within));
            }
            // (without bounds a slot past the run keeps whatever lanes: only the first n slots are
            // passed on below, and in the usual case all four share one set of live lanes)
            if constexpr (BOUNDS) {
                if ((uint32_t)g >= n) go[g] = 0;
                if (go[g] != 0) tb.visits += x_hi * 4u;
            }
        }
        if constexpr (BOUNDS) { if ((go[0] | go[1] | go[2] | go[3]) == 0) continue; }
        // (fewer than four digits left in the run: only those slots go through the stream - a slot
        // without lanes would still cost its vector instructions)
        if (n >= 4) loop_x32_masked<4, BOUNDS>(U.xq, thr, go, mk, qe, endb, full, m);
        else if (n == 3) loop_x32_masked<3, BOUNDS>(U.xq, thr, go, mk, qe, endb, full, m);
        else if (n == 2) loop_x32_masked<2, BOUNDS>(U.xq, thr, go, mk, qe, endb, full, m);
        else loop_x32_masked<1, BOUNDS>(U.xq, thr, go, mk, qe, endb, full, m);
        if constexpr (MODE == MODE_OBJ) {
            // the four digits' cheapest candidate first: mostly none of them lies within the limit
            // (a slot past the run, or without lanes, kept m = 0xFFFFFFFF)
            const uint32_t r01 = umin(__builtin_elementwise_add_sat(m[0], key4[0]), __builtin_elementwise_add_sat(m[1], key4[1]));
            const uint32_t r23 = umin(__builtin_elementwise_add_sat(m[2], key4[2]), __builtin_elementwise_add_sat(m[3], key4[3]));
            const uint32_t cand4 = __builtin_elementwise_add_sat(umin(r01, r23), k32);
            if (__builtin_amdgcn_ballot_w64(cand4 <= umin(tb.klim, klim_blk)) == 0) continue;
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t rel = __builtin_elementwise_add_sat(m[g], key4[g]);    // stays 0xFFFFFFFF if none
            if constexpr (MODE == MODE_OBJ) {
                // first of the two passes of objective mode (see loop_x); the second, rare, takes the
                // general path with the lane state of this digit
                const uint32_t cand = __builtin_elementwise_add_sat(rel, k32);
                bool want = cand <= umin(tb.klim, klim_blk);
                if ((uint32_t)g < n && __builtin_amdgcn_ballot_w64(want) != 0) {
                    // Exactly: every candidate of this pair of digits costs at least what the cheapest one
                    // does and is at most as accurate as the combination's best variant, so none scores
                    // more than this (same operations as the objective itself, which are monotone).
                    const uint32_t cost = cost_out + (cand >> U.lb);
                    const double most = __builtin_fma(-U.beta, (double)cost, an_tmax);
                    want = want & (most >= tb.obj) & (most >= U.obj_seen);
                }
                if ((uint32_t)g < n && __builtin_amdgcn_ballot_w64(want) != 0) {
                    const LaneState s1 = make_s1(d + g);
                    TileBest again = tb;
                    again.visits = 0;
                    loop_x32_obj<BOUNDS>(s1, U, 0, x_hi, full, again);
                    tb.k32 = again.k32; tb.obj = again.obj; tb.klim = again.klim;
                }
            } else {
                best_rel = best_rel < rel ? best_rel : rel;        // (a slot without lanes kept m = 0xFFFFFFFF)
            }
        }
    }
    if constexpr (MODE != MODE_OBJ) {
        const uint32_t cand = __builtin_elementwise_add_sat(best_rel, k32);
        tb.k32 = tb.k32 < cand ? tb.k32 : cand;
    }
}

// Two in-lane positions: runs of position 1, each with its masks, then its digits.
template <int MODE, bool BOUNDS, bool E01>
__device__ __forceinline__ void loop_y_masked(const LaneState& s, const Uniforms& U, uint32_t lo, uint32_t hi,
                                              uint32_t x_hi, uint64_t full, TileBest& tb)
{
#pragma clang fp contract(off)      // fp64 operations exactly as written (order: see jsv_device.h)
    const Entry JSV_CONST* ty = U.tab[1];
    const uint32_t nvx = __builtin_amdgcn_readfirstlane(U.nvx);
    uint32_t qe[MAX_XVAR];
#pragma unroll
    for (int v = 0; v < MAX_XVAR; ++v) qe[v] = U.xqe[v];
    const uint32_t endb = x_hi * (uint32_t)sizeof(QuadC);
    const uint64_t alive0 = __builtin_amdgcn_ballot_w64(s.smax <= U.sloq);
    const uint32_t thr0 = __builtin_elementwise_sub_sat(U.sloq, s.nxt[0]);
    const uint32_t room1 = __builtin_elementwise_sub_sat(U.sloq, s.nxt[1]);
    uint32_t d = lo;
    while (d < hi) {
        // a run of digits of position 1 that share their accuracy: what fix_position<1> does to the
        // accuracy state, then Eq. 13 for every variant of position 0
        const uint32_t run_end = U.yrun[d];
        const uint32_t re = run_end < hi ? run_end : hi;
        const double H = ty[d].acc * s.hin[1];
        const double sacc = E01 ? s.sacc : s.sacc + H;
        const double hin0 = __builtin_fma(U.w01, H, s.hin[0]);
        uint64_t mk[MAX_XVAR];
        uint32_t klim_blk = 0xFFFFFFFEu, clim_abs = 0xFFFFFFFFu;
        double an_tmax = 0.0;
        if constexpr (MODE == MODE_OBJ) {
            double tmax;
            variant_masks_tmax(U, nvx, hin0, sacc, mk, tmax);
            an_tmax = U.alpha_n * tmax;
            combination_limits(U, tb, s.cost_out, an_tmax, klim_blk, clim_abs);
        } else variant_masks(U, nvx, hin0, sacc, mk);
        y_batches<MODE, BOUNDS, E01>(U, s.smax, thr0, room1, alive0, s.k32, s.cost_out, d, re, mk, qe, endb, x_hi, full, tb,
            [&](uint32_t yd) { return fix_position<1>(s, U, ty[yd].lat, ty[yd].acc, 0, U.k32[1][yd]); }, klim_blk, clim_abs, an_tmax);
        d = re;
    }
}

// Three in-lane positions.  The accuracy outcome depends on the variants only, so the loops
// run by runs: for a run of position 2 (digits of one variant) and a run of position 1 the
// masks are made once and serve every pair of their digits; per digit of position 2 only its
// latency state (what fix_position<2> does to tails and keys) is formed again.  Same
// operations on the same operands as digit by digit, in another order of the candidates.
template <int MODE, bool BOUNDS, bool E01>
__device__ __forceinline__ void loop_zy_masked(const LaneState& s, const Uniforms& U0, uint32_t lo, uint32_t hi,
                                               uint32_t x_hi, uint64_t full, TileBest& tb)
{
#pragma clang fp contract(off)      // fp64 operations exactly as written (order: see jsv_device.h)
    // objective mode with bounds: the bound moves while the tile runs, run by run of position 2 (see
    // Moving; in the cost mode this loop only sees the small tiles that the pair stream leaves it,
    // where taking the bound in run by run costs more than it excludes)
    constexpr bool MOVING = BOUNDS && is_obj(MODE);
    Uniforms V = U0;
    const Uniforms& U = V;
    const Entry JSV_CONST* ty = U.tab[1];
    const Entry JSV_CONST* tz = U.tab[2];
    const uint32_t nvx = __builtin_amdgcn_readfirstlane(U.nvx);
    const uint32_t src2 = __builtin_amdgcn_readfirstlane(U.src[2] ? 1u : 0u);
    uint32_t qe[MAX_XVAR];
#pragma unroll
    for (int v = 0; v < MAX_XVAR; ++v) qe[v] = U.xqe[v];
    const uint32_t endb = x_hi * (uint32_t)sizeof(QuadC);
    const uint32_t KY = U.K[1];
    Moving mv = bound_start<MODE>(V, tb);
    uint32_t z = lo;
    while (z < hi) {
        const uint32_t zrun_end = U.zrun[z];
        const uint32_t zre = zrun_end < hi ? zrun_end : hi;
        if constexpr (MOVING) bound_take_in<MODE>(V, mv);
        // accuracy state with position 2 fixed to this variant (fix_position<2>)
        const double Hz = tz[z].acc * s.hin[2];
        const double sacc2 = src2 != 0 ? s.sacc + Hz : s.sacc;
        const double hin1 = __builtin_fma(U.w12, Hz, s.hin[1]);
        const double hin0z = __builtin_fma(U.w02, Hz, s.hin[0]);
        uint32_t y = 0;
        while (y < KY) {
            const uint32_t yre = U.yrun[y];
            // ... and position 1 to this one (fix_position<1>), then Eq. 13 per variant of position 0
            const double H = ty[y].acc * hin1;
            const double sacc = E01 ? sacc2 : sacc2 + H;
            const double hin0 = __builtin_fma(U.w01, H, hin0z);
            uint64_t mk[MAX_XVAR];
            uint32_t klim_blk = 0xFFFFFFFEu, clim_abs = 0xFFFFFFFFu;
            double an_tmax = 0.0;
            if constexpr (MODE == MODE_OBJ) {
                double tmax;
                variant_masks_tmax(U, nvx, hin0, sacc, mk, tmax);
                an_tmax = U.alpha_n * tmax;
                combination_limits(U, tb, s.cost_out, an_tmax, klim_blk, clim_abs);
            } else variant_masks(U, nvx, hin0, sacc, mk);
            for (uint32_t zd = z; zd < zre; ++zd) {
                // latency state and key with this digit of position 2 fixed
                const uint32_t tail = tz[zd].lat + s.nxt[2];
                const uint32_t smax = src2 != 0 ? umax(s.smax, tail) : s.smax;
                const uint32_t nxt1 = umax(s.nxt[1], tail & U.m12);
                const uint32_t nxt0 = umax(s.nxt[0], tail & U.m02);
                const uint32_t k32 = s.k32 + U.k32[2][zd];
                if constexpr (BOUNDS) {
                    // is any lane left that meets the latency SLO so far and stays within the cost
                    // bound with the cheapest entries of the two positions below?
                    const uint32_t fixed = s.cost_out + (k32 >> U.lb);
                    const uint32_t within = MODE == MODE_OBJ ? umin(clim_abs, U.bound) : U.bound;
                    if (__builtin_amdgcn_ballot_w64((smax <= U.sloq) & (fixed + U.min_xy_cost <= within)) == 0) continue;
                }
                const uint64_t alive0 = __builtin_amdgcn_ballot_w64(smax <= U.sloq);
                const uint32_t thr0 = __builtin_elementwise_sub_sat(U.sloq, nxt0);
                const uint32_t room1 = __builtin_elementwise_sub_sat(U.sloq, nxt1);
                y_batches<MODE, BOUNDS, E01>(U, smax, thr0, room1, alive0, k32, s.cost_out, y, yre, mk, qe, endb, x_hi, full, tb,
                    [&](uint32_t yd) {
                        const LaneState s2 = fix_position<2>(s, U, tz[zd].lat, tz[zd].acc, 0, U.k32[2][zd]);
                        return fix_position<1>(s2, U, ty[yd].lat, ty[yd].acc, 0, U.k32[1][yd]);
                    }, klim_blk, clim_abs, an_tmax);
            }
            y = yre;
        }
        if constexpr (MOVING) bound_publish<MODE>(s, V, tb, mv);
        z = zre;
    }
    if constexpr (MOVING) { tb.bound = V.bound; tb.obj_seen = V.obj_seen; }
}

// Three in-lane positions with the pair stream (cost modes, single tuples).  The slots that go
// through a record together are up to four digits of position 2 (one run: one variant, so one
// set of masks per run of position 1 serves them all), and the records are those of the pair
// stream: for the digit of position 1 at hand, position 0's candidates with that digit's key
// already in theirs.  A slot's running minimum therefore covers positions 1 and 0 together and
// stays in its register across all digits of position 1; per (digit of position 2, digit of
// position 1) only the latency threshold is formed (two vector instructions), per candidate
// the same two as everywhere.  Same tests on the same operands as digit by digit.
//
// One batch of G digits of position 2, starting at zb, against all digits of position 1 (the
// slot count is a template parameter so that the minima keep their registers over the loops).
// sacc2, hin1, hin0z: the accuracy state with position 2 fixed to the run's variant.
template <int MODE, int G, bool BOUNDS, bool E01, bool SAME_ROOM = false>
__device__ __forceinline__ void z_batch_pairs(const LaneState& s, Uniforms& U, Moving& mv, uint32_t zb, uint32_t nvx, uint32_t src2,
                                              double sacc2, double hin1, double hin0z, const uint32_t (&qe)[MAX_XVAR],
                                              uint32_t endb, uint32_t x_hi, uint64_t full, TileBest& tb)
{
#pragma clang fp contract(off)      // fp64 operations exactly as written (order: see jsv_device.h)
    // cost mode with bounds: the bound moves while the tile runs, from one run of position 1 that is
    // gone through to the next (see Moving)
    constexpr bool MOVING = BOUNDS && MODE == MODE_COST;
    const Entry JSV_CONST* ty = U.tab[1];
    const Entry JSV_CONST* tz = U.tab[2];
    const uint32_t KY = U.K[1];
    // latency state and key of each slot's digit of position 2
    uint32_t thr0[4], room1[4], k32z[4], m[4];
    uint64_t alive[4];
    uint64_t any = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint32_t zd = zb + (uint32_t)g;
        const uint32_t tail = tz[zd].lat + s.nxt[2];
        const uint32_t smax = src2 != 0 ? umax(s.smax, tail) : s.smax;
        const uint32_t nxt1 = umax(s.nxt[1], tail & U.m12);
        const uint32_t nxt0 = umax(s.nxt[0], tail & U.m02);
        k32z[g] = s.k32 + U.k32[2][zd];
        thr0[g] = __builtin_elementwise_sub_sat(U.sloq, nxt0);
        room1[g] = __builtin_elementwise_sub_sat(U.sloq, nxt1);
        m[g] = 0xFFFFFFFFu;
        bool meets = smax <= U.sloq;
        if constexpr (BOUNDS) {
            // ... and stays within the cost bound with the cheapest entries of the two positions below
            const uint32_t fixed = s.cost_out + (k32z[g] >> U.lb);
            meets = meets & (fixed + U.min_xy_cost <= U.bound);
        }
        alive[g] = __builtin_amdgcn_ballot_w64(meets);
        any |= alive[g];
    }
#pragma unroll
    for (int g = G; g < 4; ++g) { thr0[g] = 0; room1[g] = 0; k32z[g] = 0; m[g] = 0xFFFFFFFFu; alive[g] = 0; }
    if constexpr (BOUNDS) { if (any == 0) return; }
    uint32_t y = 0;
    while (y < KY) {
        const uint32_t yre = U.yrun[y];
        if constexpr (BOUNDS) {
            // The run as a whole first: with its cheapest digit and its fastest one, can any lane of any
            // slot stay within the cost bound and leave position 0 a candidate?  Mostly none can, and
            // the run is left out before its masks are made and its digits are tested one by one.
            const uint32_t rk = U.yrk[y], rl = U.yrl[y];
            uint64_t some = 0;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const uint32_t most = E01 ? umin(thr0[g], __builtin_elementwise_sub_sat(room1[g], rl)) : thr0[g];
                const uint32_t fixed = s.cost_out + ((k32z[g] + rk) >> U.lb);
                bool can = (most >= U.min_x_lat) & (fixed + U.min_x_cost <= U.bound);
                if constexpr (!E01) can = can & (rl <= room1[g]);
                some |= alive[g] & __builtin_amdgcn_ballot_w64(can);
            }
            if (some == 0) { y = yre; continue; }
        }
        if constexpr (MOVING) bound_take_in<MODE>(U, mv);
        // position 1 fixed to this run's accuracy (fix_position<1>), then Eq. 13 per variant of position 0
        const double H = ty[y].acc * hin1;
        const double sacc = E01 ? sacc2 : sacc2 + H;
        const double hin0 = __builtin_fma(U.w01, H, hin0z);
        uint64_t mk[MAX_XVAR];
        uint32_t klim_blk = 0xFFFFFFFEu, clim_abs = 0xFFFFFFFFu;
        double an_tmax = 0.0;
        if constexpr (MODE == MODE_OBJ) {
            // objective mode: the limits of this combination of variants (see combination_limits); the
            // slots' minima start afresh, so that a minimum within the limit belongs to this run
            double tmax;
            variant_masks_tmax(U, nvx, hin0, sacc, mk, tmax);
            an_tmax = U.alpha_n * tmax;
            combination_limits(U, tb, s.cost_out, an_tmax, klim_blk, clim_abs);
#pragma unroll
            for (int g = 0; g < G; ++g) m[g] = 0xFFFFFFFFu;
        } else variant_masks(U, nvx, hin0, sacc, mk);
        for (uint32_t dy = y; dy < yre; ++dy) {
            const uint32_t lat = U.ylat[dy];
            uint32_t thr[4] = {0, 0, 0, 0};
            uint64_t go[4] = {0, 0, 0, 0};
            // as in y_batches: position 1 either feeds position 0's threshold or is a source
            if constexpr (E01 && SAME_ROOM) {
                // position 2 does not feed position 1: all slots leave position 1 the same room
                const uint32_t left = __builtin_elementwise_sub_sat(room1[0], lat);
#pragma unroll
                for (int g = 0; g < G; ++g) thr[g] = umin(thr0[g], left);
            } else if constexpr (E01) {
#pragma unroll
                for (int g = 0; g < G; ++g) thr[g] = umin(thr0[g], __builtin_elementwise_sub_sat(room1[g], lat));
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                go[g] = alive[g];
                if constexpr (!E01) { thr[g] = thr0[g]; go[g] = alive[g] & __builtin_amdgcn_ballot_w64(lat <= room1[g]); }
                if constexpr (BOUNDS) {
                    const uint32_t fixed = s.cost_out + ((k32z[g] + U.yk32[dy]) >> U.lb);
                    const uint32_t within = MODE == MODE_OBJ ? umin(clim_abs, U.bound) : U.bound;
                    go[g] &= __builtin_amdgcn_ballot_w64((thr[g] >= U.min_x_lat) & (fixed + U.min_x_cost <= within));
                    if (go[g] != 0) tb.visits += x_hi * 4u;
                }
            }
            if constexpr (BOUNDS) { if ((go[0] | go[1] | go[2] | go[3]) == 0) continue; }
            loop_x32_masked<G, BOUNDS>(U.pairs + (size_t)dy * U.pair_nq, thr, go, mk, qe, endb, full, m);
            if constexpr (MODE == MODE_OBJ) {
                // First of the two passes of objective mode (see loop_x).  A slot's minimum runs over the
                // digits of position 1 since it was last reset; while it lies above the limit nothing so
                // far can matter, and once it lies within, this digit gets its second pass (its own
                // cheapest candidate is at least that minimum) and the minimum starts afresh.
                uint32_t c[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
#pragma unroll
                for (int g = 0; g < G; ++g) c[g] = __builtin_elementwise_add_sat(m[g], k32z[g]);
                const uint32_t cmin = umin(umin(c[0], c[1]), umin(c[2], c[3]));
                if (__builtin_amdgcn_ballot_w64(cmin <= umin(tb.klim, klim_blk)) == 0) continue;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    bool want = c[g] <= umin(tb.klim, klim_blk);
                    if (__builtin_amdgcn_ballot_w64(want) == 0) continue;
                    m[g] = 0xFFFFFFFFu;
                    // exactly: nothing of this pair of digits scores more than its cheapest candidate would
                    // with the combination's best accuracy (see y_batches)
                    const uint32_t cost = s.cost_out + (c[g] >> U.lb);
                    const double most = __builtin_fma(-U.beta, (double)cost, an_tmax);
                    want = want & (most >= tb.obj) & (most >= U.obj_seen);
                    if (__builtin_amdgcn_ballot_w64(want) == 0) continue;
                    const uint32_t zd = zb + (uint32_t)g;
                    const LaneState s2 = fix_position<2>(s, U, tz[zd].lat, tz[zd].acc, 0, U.k32[2][zd]);
                    const LaneState s1 = fix_position<1>(s2, U, ty[dy].lat, ty[dy].acc, 0, U.k32[1][dy]);
                    TileBest again = tb;
                    again.visits = 0;
                    loop_x32_obj<BOUNDS>(s1, U, 0, x_hi, full, again);
                    tb.k32 = again.k32; tb.obj = again.obj; tb.klim = again.klim;
                }
            }
        }
        if constexpr (MOVING) {
            // the cheapest candidate this lane has met in the tile, the slots' minima so far included
            TileBest now = tb;
#pragma unroll
            for (int g = 0; g < G; ++g) now.k32 = umin(now.k32, __builtin_elementwise_add_sat(m[g], k32z[g]));
            bound_publish<MODE>(s, U, now, mv);
        }
        y = yre;
    }
    if constexpr (MODE != MODE_OBJ) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint32_t cand = __builtin_elementwise_add_sat(m[g], k32z[g]);    // stays 0xFFFFFFFF if none
            tb.k32 = tb.k32 < cand ? tb.k32 : cand;
        }
    }
}

template <int MODE, bool BOUNDS, bool E01>
__device__ __forceinline__ void loop_zyx_pairs(const LaneState& s, const Uniforms& U, uint32_t lo, uint32_t hi,
                                               uint32_t x_hi, uint64_t full, TileBest& tb)
{
#pragma clang fp contract(off)      // fp64 operations exactly as written (order: see jsv_device.h)
    const Entry JSV_CONST* tz = U.tab[2];
    const uint32_t nvx = __builtin_amdgcn_readfirstlane(U.nvx);
    const uint32_t src2 = __builtin_amdgcn_readfirstlane(U.src[2] ? 1u : 0u);
    uint32_t qe[MAX_XVAR];
#pragma unroll
    for (int v = 0; v < MAX_XVAR; ++v) qe[v] = U.xqe[v];
    const uint32_t endb = x_hi * (uint32_t)sizeof(QuadC);
    // cost mode with bounds: the bound moves while the tile runs (see z_batch_pairs)
    constexpr bool MOVING = BOUNDS && MODE == MODE_COST;
    Uniforms V = U;
    Moving mv = bound_start<MODE>(V, tb);
    uint32_t z = lo;
    while (z < hi) {
        const uint32_t zrun_end = U.zrun[z];
        const uint32_t zre = zrun_end < hi ? zrun_end : hi;
        // accuracy state with position 2 fixed to this variant (fix_position<2>)
        const double Hz = tz[z].acc * s.hin[2];
        const double sacc2 = src2 != 0 ? s.sacc + Hz : s.sacc;
        const double hin1 = __builtin_fma(U.w12, Hz, s.hin[1]);
        const double hin0z = __builtin_fma(U.w02, Hz, s.hin[0]);
        uint32_t zb = z;
        // full batches are compiled a second time for graphs in which position 2 does not feed position 1
        if (E01 && U.m12 == 0)
            for (; zb + 4 <= zre; zb += 4) z_batch_pairs<MODE, 4, BOUNDS, E01, true>(s, V, mv, zb, nvx, src2, sacc2, hin1, hin0z, qe, endb, x_hi, full, tb);
        else
            for (; zb + 4 <= zre; zb += 4) z_batch_pairs<MODE, 4, BOUNDS, E01>(s, V, mv, zb, nvx, src2, sacc2, hin1, hin0z, qe, endb, x_hi, full, tb);
        switch (zre - zb) {
        case 3: z_batch_pairs<MODE, 3, BOUNDS, E01>(s, V, mv, zb, nvx, src2, sacc2, hin1, hin0z, qe, endb, x_hi, full, tb); break;
        case 2: z_batch_pairs<MODE, 2, BOUNDS, E01>(s, V, mv, zb, nvx, src2, sacc2, hin1, hin0z, qe, endb, x_hi, full, tb); break;
        case 1: z_batch_pairs<MODE, 1, BOUNDS, E01>(s, V, mv, zb, nvx, src2, sacc2, hin1, hin0z, qe, endb, x_hi, full, tb); break;
        default: break;
        }
        z = zre;
    }
    if constexpr (MOVING) tb.bound = V.bound;
}

template <bool W32, int MODE, bool BOUNDS>
__device__ __forceinline__ void loop_y(const LaneState& s, const Uniforms& U, uint32_t lo, uint32_t hi,
                                       uint32_t x_hi, uint64_t full, Best& best, TileBest& tb)
{
    if constexpr (W32 && !is_mix(MODE)) {
        // single tuples with few variants in position 0 (nvx is 0 for a stream of mixtures)
        // (position 1 is a source exactly when position 0, its only possible predecessor, does not feed it)
        if (U.nvx - 1u < (uint32_t)MAX_XVAR && U.src[1] == (U.m01 == 0)) {
            if (U.m01 != 0) loop_y_masked<MODE, BOUNDS, true>(s, U, lo, hi, x_hi, full, tb);
            else loop_y_masked<MODE, BOUNDS, false>(s, U, lo, hi, x_hi, full, tb);
            return;
        }
    }
    const Entry JSV_CONST* ty = U.tab[1];
    for (uint32_t d = lo; d < hi; ++d) {
        const LaneState s1 = fix_position<1>(s, U, ty[d].lat, ty[d].acc, W32 ? 0 : ty[d].key,
                                             W32 ? U.k32[1][d] : 0u);
        loop_x<W32, MODE, BOUNDS>(s1, U, 0, x_hi, full, best, tb);
    }
}

template <bool W32, int MODE, bool BOUNDS>
__device__ __forceinline__ void loop_z(const LaneState& s, const Uniforms& U, uint32_t lo, uint32_t hi,
                                       uint32_t x_hi, uint64_t full, Best& best, TileBest& tb)
{
    if constexpr (W32 && !is_mix(MODE)) {
        // single tuples with few variants in position 0: by runs of positions 2 and 1 (see loop_y for the tests)
        if (U.nvx - 1u < (uint32_t)MAX_XVAR && U.src[1] == (U.m01 == 0)) {
            // (worth it from four digits of position 2 per tile: they are the slots that share a record;
            // objective mode with bounds stays with the loops below: there the pair loop's larger
            // register set costs more in resident waves than it saves in instructions)
            if constexpr (MODE == MODE_COST || !BOUNDS) {
                if (U.pair_nq != 0 && hi - lo >= 4u) {
                    if (U.m01 != 0) loop_zyx_pairs<MODE, BOUNDS, true>(s, U, lo, hi, x_hi, full, tb);
                    else loop_zyx_pairs<MODE, BOUNDS, false>(s, U, lo, hi, x_hi, full, tb);
                    return;
                }
            }
            if (U.m01 != 0) loop_zy_masked<MODE, BOUNDS, true>(s, U, lo, hi, x_hi, full, tb);
            else loop_zy_masked<MODE, BOUNDS, false>(s, U, lo, hi, x_hi, full, tb);
            return;
        }
    }
    const Entry JSV_CONST* tz = U.tab[2];
    // with bounds and 32-bit keys: the bound moves while the tile runs, digit by digit of position 2 (see Moving)
    constexpr bool MOVING = BOUNDS && W32;
    Uniforms V = U;
    Moving mv = bound_start<MODE>(V, tb);
    for (uint32_t d = lo; d < hi; ++d) {
        if constexpr (MOVING) bound_take_in<MODE>(V, mv);
        const LaneState s2 = fix_position<2>(s, V, tz[d].lat, tz[d].acc, W32 ? 0 : tz[d].key,
                                             W32 ? U.k32[2][d] : 0u);
        if constexpr (BOUNDS) {
            // with this digit fixed, is any lane left that meets the latency SLO so far and stays
            // within the cost bound with the cheapest entries of the two positions below?
            const uint64_t fixed = W32 ? (uint64_t)(s2.cost_out + (s2.k32 >> U.lb)) : (s2.key >> U.idx_bits);
            if (__builtin_amdgcn_ballot_w64((s2.smax <= U.sloq) & (fixed + U.min_xy_cost <= V.bound)) == 0) continue;
        }
        loop_y<W32, MODE, BOUNDS>(s2, V, 0, U.K[1], x_hi, full, best, tb);
        if constexpr (MOVING) bound_publish<MODE>(s, V, tb, mv);
    }
    if constexpr (MOVING) { tb.bound = V.bound; tb.obj_seen = V.obj_seen; }
}

// One tile: 256 lanes, each a different combination of the positions >= NIN
// (decoded from the mixed-radix outer index), all looping over the same digits of
// positions < NIN.
template <int NIN, bool W32, int MODE, bool BOUNDS>
__device__ __forceinline__ void run_tile(const Graph JSV_CONST* g, const Instance JSV_CONST* in,
                                         const Entry JSV_CONST* tab, const uint32_t JSV_CONST* k32,
                                         const Quad JSV_CONST* quads, const QuadC JSV_CONST* pairs, const Entry* s_tab, uint32_t k_max, bool mix,
                                         uint64_t group, uint32_t chunk_id, uint32_t& bound, uint32_t fresh, uint32_t* bound_at,
                                         unsigned long long* best_obj_at, double& obj_seen, Best& best, uint64_t& visited)
{
#pragma clang fp contract(off)      // fp64 operations exactly as written (order: see jsv_device.h)
    const uint32_t T = g->T;
    uint64_t o = group * TILE_LANES + threadIdx.x;
    const bool live = o < in->s_out;
    if (!live) o = 0;

    // digits of the outer positions, position NIN fastest
    uint32_t dig[MAXT];
    if (in->s_out <= 0xFFFFFFFFull) {
        uint32_t o32 = (uint32_t)o;
#pragma unroll
        for (int p = NIN; p < MAXT; ++p)
            if (p < (int)T) o32 = div_by_magic(o32, in->kpos[p], in->mpos[p], &dig[p]);
    } else {
#pragma unroll
        for (int p = NIN; p < MAXT; ++p)
            if (p < (int)T) { const uint32_t K = in->K[g->task_at[p]]; dig[p] = (uint32_t)(o % K); o /= K; }
    }

    // backward recursion over the outer positions, entries gathered from LDS
    uint32_t tail[MAXT];
    double H[MAXT];
    LaneState st;
    st.smax = live ? 0u : 0xFFFFFFFFu;      // a dead lane can never meet the latency SLO
    st.sacc = 0.0; st.key = 0; st.k32 = 0;
    const uint32_t src_mask = g->src_mask, sink_mask = g->sink_mask;
#pragma unroll
    for (int p = MAXT - 1; p >= NIN; --p) {
        if (p < (int)T) {
            const Entry* e = s_tab + in->rowpos[p] + dig[p];
            const uint32_t lat = e->lat;
            const double acc = e->acc;
            st.key += e->key;
            uint32_t mx = 0;
            double hs = 0.0;
            const uint32_t succ = g->succ[p];
#pragma unroll
            for (int s = MAXT - 1; s > p; --s)
                if ((succ >> s) & 1u) { mx = umax(mx, tail[s]); hs = __builtin_fma(g->w[p][s], H[s], hs); }
            tail[p] = lat + mx;
            H[p] = acc * (((sink_mask >> p) & 1u) ? g->u[p] : hs);
            if ((src_mask >> p) & 1u) { st.smax = umax(st.smax, tail[p]); st.sacc = st.sacc + H[p]; }
        }
    }
    // what the outer positions contribute to the recursions of positions < NIN
#pragma unroll
    for (int p = 0; p < 3; ++p) { st.nxt[p] = 0; st.hin[p] = g->u[p]; }     // u(p) = 0 unless p is a sink
#pragma unroll
    for (int p = 0; p < NIN; ++p) {
        const uint32_t succ = g->succ[p];
#pragma unroll
        for (int s = MAXT - 1; s >= NIN; --s)
            if ((succ >> s) & 1u) { st.nxt[p] = umax(st.nxt[p], tail[s]); st.hin[p] = __builtin_fma(g->w[p][s], H[s], st.hin[p]); }
    }

    Uniforms U;
#pragma unroll
    for (int p = 0; p < 3; ++p) {
        const uint32_t row = in->rowpos[p < NIN ? p : 0];
        U.tab[p] = tab + row;
        U.k32[p] = k32 + row;
        U.K[p] = in->kpos[p < NIN ? p : 0];
        U.src[p] = (src_mask >> p) & 1u;
    }
    U.quads = quads;
    U.m01 = 0u - ((g->succ[0] >> 1) & 1u); U.m02 = 0u - ((g->succ[0] >> 2) & 1u); U.m12 = 0u - ((g->succ[1] >> 2) & 1u);
    U.w01 = g->w[0][1]; U.w02 = g->w[0][2]; U.w12 = g->w[1][2];
    U.sloq = in->sloq;
    U.min_x_lat = in->min_x_lat;
    U.min_x_cost = in->min_x_cost;
    U.min_xy_cost = in->min_xy_cost;
    // (with bounds: what the instance's bound has become since the wave last looked - the load was
    // issued before the tile's set-up, so it is there by now)
    if constexpr (BOUNDS) {
        const uint32_t f = (uint32_t)__builtin_amdgcn_readfirstlane((int)fresh);
        bound = f < bound ? f : bound;
    }
    U.bound = bound;
    U.bound_at = bound_at;
    U.best_obj_at = best_obj_at;
    U.obj_seen = MODE == MODE_OBJ ? obj_seen : -__builtin_inf();
    U.slo_raw = in->slo_raw;
    U.idx_bits = in->idx_bits; U.lb = in->lb; U.capacity = g->capacity;
    U.alpha_n = in->alpha_n; U.beta = in->beta;
    U.alpha = in->alpha; U.inv_beta = in->inv_beta; U.mix = mix;
    U.nvx = in->nvx; U.xacc = in->xacc; U.xqe = in->xqe; U.xq = (const QuadC JSV_CONST*)(quads + quadc_offset(k_max));
    U.ylat = (const uint32_t JSV_CONST*)(quads + yrec_offset(k_max));
    U.yk32 = U.ylat + ydigit_words(k_max);
    U.yrun = U.yk32 + ydigit_words(k_max);
    U.zrun = U.yrun + ydigit_words(k_max);
    U.yrk = U.zrun + ydigit_words(k_max);
    U.yrl = U.yrk + ydigit_words(k_max);
    U.pairs = pairs; U.pair_nq = in->pair_nq;
    st.cost_out = (uint32_t)(st.key >> in->idx_bits);
    // Cost as a bound: `bound` is S_avail (Eq. 8) or, in the cost modes, the cost of a candidate
    // already found that meets both SLOs, whichever is lower.  A lane whose fixed positions plus
    // the cheapest entries of the in-lane positions cost more holds neither a candidate within
    // S_avail nor one cheaper than what is known; it sits out like a lane that cannot meet the
    // latency SLO.  Candidates as cheap as the bound stay in (the lowest index wins among them).
    if constexpr (BOUNDS) {
        if ((uint64_t)st.cost_out + in->min_in_cost > bound) st.smax = 0xFFFFFFFFu;
        if (__builtin_amdgcn_ballot_w64(st.smax <= U.sloq) == 0) return;     // nothing left for this wave
    }

    // extent of the innermost loop (quads of the stream, or digits) and of the chunked loop
    const uint32_t x_all = W32 ? in->nq : U.K[0];
    const uint32_t Ko = NIN == 1 ? x_all : U.K[NIN - 1];
    const uint32_t lo = chunk_id * in->chunk;
    const uint32_t hi = lo + in->chunk < Ko ? lo + in->chunk : Ko;
    TileBest tb;
    // (objective mode, 32-bit keys: the tile's best starts at the objective the lane already holds, with
    // no key - a candidate must reach that objective to be noted, and ties are settled on the full
    // keys after the tile)
    tb.k32 = 0xFFFFFFFFu; tb.obj = (is_obj(MODE) && W32) ? best.obj : -__builtin_inf(); tb.visits = 0;
    tb.klim = 0xFFFFFFFEu; tb.bound = U.bound; tb.obj_seen = U.obj_seen;
    if constexpr (is_obj(MODE) && W32) tb.klim = key_limit(U, st.cost_out, best.obj, U.alpha);
    const uint64_t full = __builtin_amdgcn_read_exec();     // the loops below run convergent
    if constexpr (NIN == 3) loop_z<W32, MODE, BOUNDS>(st, U, lo, hi, x_all, full, best, tb);
    else if constexpr (NIN == 2) loop_y<W32, MODE, BOUNDS>(st, U, lo, hi, x_all, full, best, tb);
    else loop_x<W32, MODE, BOUNDS>(st, U, lo, hi, full, best, tb);
    if (BOUNDS || U.mix) visited += tb.visits;
    bound = tb.bound;
    if constexpr (MODE == MODE_OBJ) obj_seen = tb.obj_seen;

    if constexpr (W32) {
        // the lane's 32-bit winner of this tile -> its full (cost, index) key; only where some lane's
        // winner can replace what the lane holds (as cheap, or with as good an objective: the index
        // decides between equals), which after the first tiles is rare
        const bool hit = tb.k32 != 0xFFFFFFFFu;
        bool may;
        if constexpr (is_obj(MODE)) may = hit && tb.obj >= best.obj;
        else may = hit && (uint64_t)st.cost_out + (tb.k32 >> in->lb) <= (best.key >> in->idx_bits);
        if (__builtin_amdgcn_ballot_w64(may) == 0) return;
        uint32_t r = hit ? (tb.k32 & ((1u << in->lb) - 1u)) : 0u;
        uint64_t k = st.key;
#pragma unroll
        for (int a = 0; a < NIN; ++a) {
            const uint32_t p = in->ord[a];
            uint32_t d;
            r = div_by_magic(r, in->kpos[p], in->mpos[p], &d);
            k += s_tab[in->rowpos[p] + d].key;
        }
        if constexpr (is_obj(MODE)) {
            if (hit && better(tb.obj, k, best.obj, best.key)) { best.obj = tb.obj; best.key = k; }
        } else {
            best.key = (hit && k < best.key) ? k : best.key;
        }
    }
}

// A block's result for one instance: its lanes' best reduced over the block.
template <bool OBJ>
__device__ __forceinline__ void flush_block(const Plan& pl, uint32_t inst, const Best& best, uint64_t* s_key, double* s_obj)
{
    if constexpr (OBJ) {
        const Best b = block_best(best, s_key, s_obj);
        if (threadIdx.x == 0) {
            pl.partial[(size_t)inst * pl.grid + blockIdx.x] = b.key;
            pl.partial_obj[(size_t)inst * pl.grid + blockIdx.x] = b.obj;
        }
    } else {
        const uint64_t m = block_min(best.key, s_key);
        if (threadIdx.x == 0) pl.partial[(size_t)inst * pl.grid + blockIdx.x] = m;
    }
}

// Persistent grid sized to what fits on the chip at once; a block starts with the run of
// tiles that is its own by its index and then draws batches from one atomic counter (see
// STATIC_ONLY_TILES_PER_BLOCK above), so uneven tiles even out without the counter being
// asked tile by tile.  Tiles are ordered by instance, a block's own run lies before everything
// the counter hands out, and the counter only grows: a block meets the instances in
// ascending order; it keeps one running minimum per lane and reduces it (wave, then block)
// only when the instance changes.  Every block ends when its own run is done and no batches
// are handed out, or with the first ticket at or past the total.
template <int MODE, bool BOUNDS>
__global__ void __launch_bounds__(256) enumerate_kernel(Plan pl)
{
    constexpr bool OBJ = is_obj(MODE);
    // the per-instance cost limit is read and lowered with bounds on, and in objective mode also
    // without them: there it only decides where the objective itself needs evaluating
    constexpr bool SHARE = BOUNDS || OBJ;
    extern __shared__ __attribute__((aligned(32))) unsigned char smem_raw[];
    Entry* s_tab = (Entry*)smem_raw;
    __shared__ uint64_t s_red[4];
    __shared__ double s_red_obj[4];
    __shared__ unsigned long long s_tile;

    const Instance JSV_CONST* insts = as_uniform((const Instance*)pl.inst);
    const Graph JSV_CONST* graphs = as_uniform(pl.graphs);
    const uint64_t total = as_uniform((const SummaryRec*)pl.summary)->total_tiles;
    // both variants are launched when bounds are on; the scan has chosen which one works
    if ((as_uniform((const SummaryRec*)pl.summary)->bounded != 0) != BOUNDS) return;
    const uint32_t tk = pl.t_max * pl.k_max;

    uint32_t cur = 0xFFFFFFFFu;     // instance whose tables are in LDS
    uint32_t scan = 0;              // instance of the current tile
    uint64_t scan_end = 0;          // first tile behind that instance
    Best best;
    best.key = NO_KEY; best.obj = -__builtin_inf();
    uint64_t visited = 0;           // wave-uniform
    uint32_t bound_seen = 0xFFFFFFFFu;      // cost bound of instance `cur` as last read or lowered by this wave
    double obj_seen = -__builtin_inf();     // objective mode: best objective of instance `cur` that this wave knows of
    const uint32_t own = as_uniform((const SummaryRec*)pl.summary)->own_tiles;
    const uint32_t rounds = as_uniform((const SummaryRec*)pl.summary)->own_rounds;
    const uint32_t batch = as_uniform((const SummaryRec*)pl.summary)->batch_tiles;
    const uint64_t* begins = pl.tile_begin;
    // rounds of own runs first (round r: the run that starts at (r * blocks + block) * own; see below),
    // then batches from the counter
    uint32_t round = 0;
    uint64_t tile = (uint64_t)blockIdx.x * own;
    uint64_t tile_end = rounds != 0 ? tile + own : tile;
    for (;; ++tile) {
        if (tile >= tile_end) {
            ++round;
            if (round < rounds) {
                // (where all tiles go out by index, shifted by one block per round: with an even grid and
                // two chunks per group a block would otherwise meet the same chunk every round)
                uint32_t slot = blockIdx.x + (batch == 0 ? round : 0u);
                if (slot >= gridDim.x) slot %= gridDim.x;
                tile = ((uint64_t)round * gridDim.x + slot) * own;
                tile_end = tile + own;
            } else {
                if (batch == 0) break;                    // everything was shared out by index
                __syncthreads();                          // everyone has read the last ticket
                if (threadIdx.x == 0) s_tile = atomicAdd(&pl.summary->next_tile, (unsigned long long)batch);
                __syncthreads();
                const unsigned long long ticket = s_tile;
                tile = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(ticket >> 32)) << 32) |
                       (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)ticket);
                tile_end = tile + batch;
            }
        }
        if (tile >= total) break;
        if (tile >= scan_end) {
            // the instance that holds this tile: the last one that begins at or before it
            uint32_t lo = 0, hi = pl.n_inst;
            while (hi - lo > 1) {
                const uint32_t mid = (lo + hi) >> 1;
                if (as_uniform(begins)[mid] <= tile) lo = mid; else hi = mid;
            }
            scan = lo;
            scan_end = insts[scan].tile_begin + insts[scan].tiles;
        }
        if (scan != cur) {
            if (cur != 0xFFFFFFFFu) {
                flush_block<OBJ>(pl, cur, best, s_red, s_red_obj);
            }
            __syncthreads();
            const Entry* src = pl.entries + (size_t)scan * tk;
            const uint4* s4 = (const uint4*)src;
            uint4* d4 = (uint4*)s_tab;
            for (uint32_t k = threadIdx.x; k < tk * 2; k += blockDim.x) d4[k] = s4[k];
            __syncthreads();
            cur = scan;
            best.key = NO_KEY; best.obj = -__builtin_inf();
            if constexpr (SHARE)
                bound_seen = (uint32_t)__builtin_amdgcn_readfirstlane(
                    (int)__hip_atomic_load(pl.bound + cur, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            if constexpr (MODE == MODE_OBJ) {
                const unsigned long long ob = __hip_atomic_load(pl.best_obj + cur, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                obj_seen = from_ordered_bits(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(ob >> 32)) << 32) |
                                             (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)ob));
            }
        }
        const Instance JSV_CONST* in = insts + cur;
        const Graph JSV_CONST* g = graphs + in->problem;
        const Entry JSV_CONST* tab = as_uniform((const Entry*)pl.entries) + (size_t)cur * tk;
        const uint32_t JSV_CONST* k32 = as_uniform((const uint32_t*)pl.k32) + (size_t)cur * tk;
        const Quad JSV_CONST* quads = as_uniform((const Quad*)pl.quads) + (size_t)cur * quad_stride(pl.k_max);
        const QuadC JSV_CONST* pairs = as_uniform((const QuadC*)pl.pairs) + (size_t)cur * (pl.pair_cap + 1);
        const uint32_t local = (uint32_t)(tile - in->tile_begin);      // an instance has fewer than 2^31 tiles
        const uint32_t n_chunks = in->n_chunks;
        uint32_t chunk_id = 0, group = local;
        if (n_chunks != 1) { group = local / n_chunks; chunk_id = local - group * n_chunks; }
        // The tile works with the instance's cost bound as this wave knows it; a stale (higher)
        // value only excludes less.  What other blocks have made of it meanwhile is fetched now and
        // taken in after the tile's set-up (with bounds) and after the tile, so that nobody waits for
        // the load.
        uint32_t bound = bound_seen;
        uint32_t fresh = 0xFFFFFFFFu;
        if constexpr (SHARE) fresh = __hip_atomic_load(pl.bound + cur, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned long long fresh_obj = 0;
        if constexpr (MODE == MODE_OBJ) fresh_obj = __hip_atomic_load(pl.best_obj + cur, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t key_before = best.key;
        const double obj_before = best.obj;
        if (in->use32) {
            switch (in->n_in) {
            case 3: run_tile<3, true, MODE, BOUNDS>(g, in, tab, k32, quads, pairs, s_tab, pl.k_max, pl.mix != 0, group, chunk_id, bound, fresh, pl.bound + cur, pl.best_obj + cur, obj_seen, best, visited); break;
            case 2: run_tile<2, true, MODE, BOUNDS>(g, in, tab, k32, quads, pairs, s_tab, pl.k_max, pl.mix != 0, group, chunk_id, bound, fresh, pl.bound + cur, pl.best_obj + cur, obj_seen, best, visited); break;
            default: run_tile<1, true, MODE, BOUNDS>(g, in, tab, k32, quads, pairs, s_tab, pl.k_max, pl.mix != 0, group, chunk_id, bound, fresh, pl.bound + cur, pl.best_obj + cur, obj_seen, best, visited); break;
            }
        } else {
            switch (in->n_in) {
            case 3: run_tile<3, false, MODE, BOUNDS>(g, in, tab, k32, quads, pairs, s_tab, pl.k_max, pl.mix != 0, group, chunk_id, bound, fresh, pl.bound + cur, pl.best_obj + cur, obj_seen, best, visited); break;
            case 2: run_tile<2, false, MODE, BOUNDS>(g, in, tab, k32, quads, pairs, s_tab, pl.k_max, pl.mix != 0, group, chunk_id, bound, fresh, pl.bound + cur, pl.best_obj + cur, obj_seen, best, visited); break;
            default: run_tile<1, false, MODE, BOUNDS>(g, in, tab, k32, quads, pairs, s_tab, pl.k_max, pl.mix != 0, group, chunk_id, bound, fresh, pl.bound + cur, pl.best_obj + cur, obj_seen, best, visited); break;
            }
        }
        if constexpr (SHARE) {
            const uint32_t other = (uint32_t)__builtin_amdgcn_readfirstlane((int)fresh);
            bound_seen = other < bound_seen ? other : bound_seen;
            bound_seen = bound < bound_seen ? bound : bound_seen;       // lowered while the tile ran
            if constexpr (MODE == MODE_OBJ) {
                const double oo = from_ordered_bits(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(fresh_obj >> 32)) << 32) |
                                                    (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)fresh_obj));
                obj_seen = oo > obj_seen ? oo : obj_seen;
            }
            // Did a lane of this wave find something better in this tile?  Then the bound may drop
            // for every block working on the instance.
            const bool improved = __builtin_amdgcn_ballot_w64((best.key != key_before) | (best.obj != obj_before)) != 0;
            if (improved) {
                uint32_t wc = 0xFFFFFFFFu;
                if constexpr (!is_obj(MODE)) {
                    // cost modes: nothing costlier than a candidate that meets both SLOs can be the answer
                    const uint32_t c = best.key == NO_KEY ? 0xFFFFFFFFu : (uint32_t)(best.key >> in->idx_bits);
                    wc = (uint32_t)wave_min((uint64_t)c);
                } else {
                    // Eq. 14: A_obj <= 1, so a candidate of cost c scores at most alpha - beta*c.  With an
                    // objective o already reached, nothing costlier than (alpha - o)/beta can match it;
                    // one unit of slack keeps the test clear of rounding and of equal objectives.
                    const Best wb = wave_best(best);
                    if constexpr (MODE == MODE_OBJ) {
                        if (wb.key != NO_KEY && wb.obj > obj_seen) {
                            obj_seen = wb.obj;
                            if ((threadIdx.x & 63u) == 0) atomicMax(pl.best_obj + cur, ordered_bits(wb.obj));
                        }
                    }
                    if (wb.key != NO_KEY && in->beta > 1e-9 * (in->alpha + 1.0)) {     // else rounding could reach a unit of cost
                        const double lim = (in->alpha - wb.obj) / in->beta;
                        if (lim >= 0.0 && lim < 2147483000.0) wc = (uint32_t)lim + 1u;
                    }
                }
                if (wc < bound_seen) {
                    bound_seen = wc;
                    if ((threadIdx.x & 63u) == 0) atomicMin(pl.bound + cur, wc);
                }
            }
        }
    }
    if (cur != 0xFFFFFFFFu) {
        flush_block<OBJ>(pl, cur, best, s_red, s_red_obj);
    }
    // (the plain enumeration of single tuples visits everything: the host reports the space;
    // the latency-sorted stream of mixture mode ends early, so its entries are counted)
    if (BOUNDS || pl.mix != 0)
        if ((threadIdx.x & 63u) == 0 && visited != 0) atomicAdd(&pl.summary->visited, (unsigned long long)visited);
}

// ---- scoring of one assignment (finalize, eval and the plan kernel's first bound) -----------
// dig[t]: digit of task id t in its surviving list.
__device__ Score score_digits(const Graph* g, const Instance* in, const Entry* entries, uint32_t k_max,
                              const uint32_t* dig)
{
#pragma clang fp contract(off)      // fp64 operations exactly as written (order: see jsv_device.h)
    uint32_t tail[MAXT];
    double H[MAXT];
    const uint32_t T = g->T;
    uint64_t cost = 0;
    uint32_t crit = 0;
    double raw = 0.0;
    for (int p = (int)T - 1; p >= 0; --p) {
        const uint32_t t = g->task_at[p];
        const Entry* e = entries + (size_t)t * k_max + dig[t];
        uint32_t mx = 0;
        double hs = 0.0;
        for (int s = (int)T - 1; s > p; --s)
            if ((g->succ[p] >> s) & 1u) { mx = umax(mx, tail[s]); hs = __builtin_fma(g->w[p][s], H[s], hs); }
        tail[p] = e->lat + mx;
        const double inner = ((g->sink_mask >> p) & 1u) ? g->u[p] : hs;
        cost += e->cost;
        if (p == 0) {                       // always a source; joins the sum by one fma
            crit = umax(crit, tail[0]);
            raw = __builtin_fma(e->acc, inner, raw);
        } else {
            H[p] = e->acc * inner;
            if ((g->src_mask >> p) & 1u) { crit = umax(crit, tail[p]); raw = raw + H[p]; }
        }
    }
    Score sc;
    const uint64_t lat = (uint64_t)g->q * crit;
    sc.latency = lat > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)lat;
    sc.cost = cost > 0x7FFFFFFFull ? 0x7FFFFFFFu : (uint32_t)cost;
    sc.accuracy = raw / g->amax;
    sc.mask = 0;
    if (lat <= in->slo_l) sc.mask |= 1;
    if (raw >= in->slo_raw) sc.mask |= 2;               // Eq. 13, the test the enumeration applies
    if (g->capacity == 0 || cost <= g->capacity) sc.mask |= 4;
    return sc;
}

// ---- finalize ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) finalize_kernel(Plan pl)
{
    __shared__ uint64_t s_red[4];
    __shared__ double s_red_obj[4];
    // instance record, graph and the winner's entries are staged in LDS by all threads, so that
    // the one thread that rescores the winner does not wait for memory load by load
    __shared__ __attribute__((aligned(16))) Instance s_in;
    __shared__ __attribute__((aligned(16))) Graph s_g;
    __shared__ __attribute__((aligned(16))) Entry s_ent[MAXT];
    static_assert(sizeof(Instance) % 8 == 0 && sizeof(Graph) % 8 == 0, "staged by 8-byte words");
    const uint32_t i = blockIdx.x;
    {
        const uint64_t* src = (const uint64_t*)(pl.inst + i);
        uint64_t* dst = (uint64_t*)&s_in;
        for (uint32_t k = threadIdx.x; k < sizeof(Instance) / 8; k += blockDim.x) dst[k] = src[k];
    }
    uint64_t m = NO_KEY;
    if (pl.objective) {
        Best v; v.key = NO_KEY; v.obj = -__builtin_inf();
        for (uint32_t b = threadIdx.x; b < pl.grid; b += blockDim.x) {
            Best o; o.key = pl.partial[(size_t)i * pl.grid + b]; o.obj = pl.partial_obj[(size_t)i * pl.grid + b];
            v = pick(v, o);
        }
        m = block_best(v, s_red, s_red_obj).key;
    } else {
        for (uint32_t b = threadIdx.x; b < pl.grid; b += blockDim.x)
            m = umin64(m, pl.partial[(size_t)i * pl.grid + b]);
        m = block_min(m, s_red);
    }
    const Instance* in = &s_in;          // complete: block_min / block_best synchronise
    {
        const uint64_t* src = (const uint64_t*)(pl.graphs + in->problem);
        uint64_t* dst = (uint64_t*)&s_g;
        for (uint32_t k = threadIdx.x; k < sizeof(Graph) / 8; k += blockDim.x) dst[k] = src[k];
    }
    const Graph* g = &s_g;
    __shared__ uint32_t s_last_block;
    // the winner's digits: one 64-bit divide per task, by one thread per task
    __shared__ uint64_t s_win;
    __shared__ uint32_t s_dig[MAXT];
    if (threadIdx.x == 0) s_win = m;
    __syncthreads();
    m = s_win;
    const bool have = m != NO_KEY && !(in->flags & (F_OVERFLOW | F_EMPTY));
    const uint64_t idx = in->idx_bits ? (m & ((1ull << in->idx_bits) - 1)) : 0;
    if (have && threadIdx.x < g->T) {
        const uint32_t t = threadIdx.x;
        const uint32_t d = (uint32_t)((idx / in->stride[t]) % in->K[t]);
        s_dig[t] = d;
        s_ent[t] = pl.entries[((size_t)i * pl.t_max + t) * pl.k_max + d];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
    ResultRec* r = pl.results + i;
    r->index = NO_KEY; r->full_index = NO_KEY; r->evaluated = in->space;
    r->accuracy = 0.0; r->latency_us = 0; r->cost_units = 0x7FFFFFFF; r->feasible = 0; r->objective = 0.0;
    r->flags = in->flags;
    for (int t = 0; t < MAXT; ++t) { r->choice[t] = 0; r->replicas[t] = 0; r->choice2[t] = 0; r->replicas2[t] = 0; }
    if (have) {
        // (the staged entries stand in for the table: one entry per task, digit 0)
        uint32_t zero[MAXT];
        for (int t = 0; t < MAXT; ++t) zero[t] = 0;
        const Score sc = score_digits(g, in, s_ent, 1, zero);
        // The rescoring repeats the enumeration's latency and accuracy tests operation by
        // operation, so only the capacity bit (Eq. 8, applied to the minimum) can be missing.  A
        // winner that fails one of the other two would mean the two disagree: reported as an
        // error, never as "infeasible".
        if ((sc.mask & 3) != 3) r->flags |= F_MISMATCH;
        if (sc.mask == 7) {
            r->index = idx; r->feasible = 1;
            r->accuracy = sc.accuracy; r->latency_us = sc.latency; r->cost_units = (int32_t)sc.cost;
            r->objective = in->alpha * sc.accuracy - in->beta * (double)sc.cost;
            uint64_t full = 0;
            bool over = false;
            for (int t = (int)g->T - 1; t >= 0; --t) {
                const Entry* e = s_ent + t;
                r->choice[t] = (uint16_t)e->choice;
                r->replicas[t] = e->rep;
                r->choice2[t] = 0xFFFF;
                if (pl.mix) {
                    r->choice2[t] = (uint16_t)(e->choice >> 16);
                    r->replicas[t] = e->rep & 0xFFFFu; r->replicas2[t] = e->rep >> 16;
                    over = true;                     // no fixed-size full space in mixture mode
                }
                if (__umul64hi(full, g->C) != 0) over = true;
                const uint64_t f2 = full * g->C + (e->choice & 0xFFFFu);
                if (f2 < full * g->C) over = true;
                full = f2;
                if (full == NO_KEY) over = true;
            }
            r->full_index = over ? NO_KEY : full;
        }
    }
    // the last block to finish writes the sweep summary
    __threadfence();
    s_last_block = (atomicAdd(&pl.summary->done_count, 1u) == pl.n_inst - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last_block) return;
    __threadfence();
    // feasible level with the largest demand, first position on equal demands: maximum of
    // (demand << 32) | (0xFFFFFFFF - position); 0 = none (demands are > 0)
    uint64_t v = 0;
    uint32_t any = 0;
    for (uint32_t k = threadIdx.x; k < pl.n_inst; k += blockDim.x) {
        const volatile ResultRec* rk = pl.results + k;
        any |= rk->flags;
        if (rk->feasible) {
            const uint64_t cand = ((uint64_t)pl.inst[k].demand << 32) | (0xFFFFFFFFu - k);
            v = cand > v ? cand : v;
        }
    }
    __shared__ uint32_t s_any;
    if (threadIdx.x == 0) s_any = 0;
    __syncthreads();
    if (any) atomicOr(&s_any, any);
    v = ~block_min(~v, s_red);           // maximum over the block, valid in thread 0
    if (threadIdx.x == 0) {
        pl.summary->best_level = v ? (int32_t)(0xFFFFFFFFu - (uint32_t)v) : -1;
        pl.summary->max_demand = (uint32_t)(v >> 32);
        pl.summary->any_flags = s_any;
    }
}

// ---- eval -------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) eval_kernel(Plan pl, const uint64_t* index, uint32_t n,
                                                   uint32_t* latency, uint32_t* replicas, int32_t* cost,
                                                   double* accuracy, uint8_t* mask, uint32_t* bad)
{
    const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n) return;
    const Instance* in = pl.inst;
    const Graph* g = pl.graphs + in->problem;
    const uint64_t idx = index[k];
    if (idx >= in->space) { atomicOr(bad, 1u); return; }
    uint32_t dig[MAXT];
    for (uint32_t t = 0; t < g->T; ++t) dig[t] = (uint32_t)((idx / in->stride[t]) % in->K[t]);
    const Score sc = score_digits(g, in, pl.entries, pl.k_max, dig);
    latency[k] = sc.latency; cost[k] = (int32_t)sc.cost; accuracy[k] = sc.accuracy; mask[k] = sc.mask;
    for (uint32_t t = 0; t < g->T; ++t)
        replicas[(size_t)k * g->T + t] = pl.entries[(size_t)t * pl.k_max + dig[t]].rep;
}

// ---- launch wrappers (called from the host planner) -------------------------------------------
size_t prune_lds_bytes(uint32_t c_max) { return (size_t)c_max * (8 + 4 + 4 + 4 + 1 + 1) + 16; }
size_t mix_lds_bytes(uint32_t c_max) { return (size_t)c_max * (8 + 8 + 4 + 4 + 4 + 4 + 1) + 16; }
size_t enumerate_lds_bytes(uint32_t t_max, uint32_t k_max) { return (size_t)t_max * k_max * sizeof(Entry); }

hipError_t launch_prune_plan_scan(const Plan& pl, hipStream_t stream)
{
    if (pl.mix)
        hipLaunchKernelGGL(mix_kernel, dim3(pl.n_inst * pl.t_max), dim3(MIX_THREADS), mix_lds_bytes(pl.c_max), stream, pl);
    else
        hipLaunchKernelGGL(prune_kernel, dim3(pl.n_inst * pl.t_max), dim3(256), prune_lds_bytes(pl.c_max), stream, pl);
    hipLaunchKernelGGL(plan_kernel, dim3(pl.n_inst), dim3(256), 0, stream, pl);
    return hipGetLastError();
}

// The instantiation a plan runs: objective mode, mixture mode or plain cheapest-feasible, each
// with or without the bulk exclusion by bounds.
using EnumerateFn = void (*)(Plan);
static EnumerateFn enumerate_entry(int mode, bool bounds)
{
    switch (mode) {
    case MODE_OBJ: return bounds ? enumerate_kernel<MODE_OBJ, true> : enumerate_kernel<MODE_OBJ, false>;
    case MODE_MIX: return bounds ? enumerate_kernel<MODE_MIX, true> : enumerate_kernel<MODE_MIX, false>;
    case MODE_MIXOBJ: return bounds ? enumerate_kernel<MODE_MIXOBJ, true> : enumerate_kernel<MODE_MIXOBJ, false>;
    default:       return bounds ? enumerate_kernel<MODE_COST, true> : enumerate_kernel<MODE_COST, false>;
    }
}

int enumerate_mode(bool objective, bool mixtures)
{
    return objective ? (mixtures ? MODE_MIXOBJ : MODE_OBJ) : mixtures ? MODE_MIX : MODE_COST;
}

// Blocks of the enumeration kernel that are resident per CU with this much LDS.  With bounds on
// both variants are launched with one grid (launch_enumerate) and the figure is that of the
// variant with bounds, which does the work in every search large enough for the grid to matter;
// where the device picks the plain variant after all, blocks beyond what is resident simply
// start later (no block ever waits for another).
hipError_t enumerate_blocks_per_cu(uint32_t t_max, uint32_t k_max, int mode, bool bounds, int* blocks)
{
    const size_t lds = enumerate_lds_bytes(t_max, k_max);
    int wanted = 0;
    for (int b = 0; b <= (bounds ? 1 : 0); ++b) {
        const void* fn = (const void*)enumerate_entry(mode, b != 0);
        if (lds > 32 * 1024) {      // beyond the default dynamic limit: ask for it explicitly
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        int n = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, fn, TILE_LANES, lds);
        if (e != hipSuccess) return e;
        if (n < 1) { *blocks = 0; return hipSuccess; }      // (a variant that does not fit at all)
        wanted = n;                                         // the last one asked: with bounds, that variant
    }
    *blocks = wanted;
    return hipSuccess;
}

hipError_t launch_enumerate(const Plan& pl, hipStream_t stream)
{
    // With bounds on, both variants go out and the one the scan did not choose returns at once
    // (the choice depends on the tile count, which only the device knows at this point).
    const int mode = enumerate_mode(pl.objective != 0, pl.mix != 0);
    const size_t lds = enumerate_lds_bytes(pl.t_max, pl.k_max);
    hipLaunchKernelGGL(enumerate_entry(mode, false), dim3(pl.grid), dim3(TILE_LANES), lds, stream, pl);
    if (pl.bounds)
        hipLaunchKernelGGL(enumerate_entry(mode, true), dim3(pl.grid), dim3(TILE_LANES), lds, stream, pl);
    return hipGetLastError();
}

hipError_t launch_finalize(const Plan& pl, hipStream_t stream)
{
    hipLaunchKernelGGL(finalize_kernel, dim3(pl.n_inst), dim3(256), 0, stream, pl);
    return hipGetLastError();
}

hipError_t launch_eval(const Plan& pl, const uint64_t* index, uint32_t n, uint32_t* latency,
                       uint32_t* replicas, int32_t* cost, double* accuracy, uint8_t* mask,
                       uint32_t* bad, hipStream_t stream)
{
    hipLaunchKernelGGL(eval_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, pl, index, n, latency,
                       replicas, cost, accuracy, mask, bad);
    return hipGetLastError();
}

}  // namespace jsv
