// Device-side data layout shared by the host planner and the HIP kernels.
//
// Positions.  Tasks are handled in a topological order fixed by the host
// (Kahn's algorithm, lowest task id first).  "Position" p means the place of a
// task in that order: p = 0 is a source.  The kernels evaluate the critical
// path (Eq. 3) and the accuracy (Eq. 11, 12) by a backward recursion over
// positions, from the sinks towards the sources:
//
//   tail(p) = L(p) + max over successors s of tail(s)            latency to the end
//   H(p)    = a(p) * ( u(p)                     if p is a sink
//                      sum_s w(p,s) * H(s)      otherwise )      accuracy mass
//   latency  = q * max over sources of tail,   A_raw = sum over sources of H
//
// with w(p,s) the share of p among the predecessors of s and u(p) the share of
// sink p among all sinks (both from the per-task demand multipliers).  Summed
// over sources this is exactly sum_p f_p * prod_{t in p} a_t of Eq. 12.
//
// One order of fp64 operations, used wherever A_raw is formed (host: A_max; device: the
// enumeration, the rescoring of the winner, jsv_eval_candidates), so that the same assignment
// always yields the same bits and the accuracy test of Eq. 13 has one outcome:
//   positions are visited from T-1 down to 0;
//   sum_s w(p,s)*H(s) starts at +0.0 and takes the successors in DESCENDING position, one fma
//     each:  hs = fma(w(p,s), H(s), hs);
//   H(p) = a(p) * (u(p) or hs), one rounded product;
//   A_raw starts at +0.0 and takes the sources in descending position, one rounded add each,
//     except position 0 (always a source, always last), which joins as  fma(a(0), hs(0), A_raw);
//   Eq. 13 is tested as  A_raw >= SLO_a * A_max  (the product rounded once, on the host).
// Descending successor order is what lets a lane hoist the part of hs that comes from the
// positions it holds fixed and add the looped positions (2, then 1) afterwards.
#pragma once
#include <stdint.h>

namespace jsv {

constexpr int MAXT = 16;          // tasks per graph
constexpr int MAXC = 2048;        // choices per task
constexpr int TILE_LANES = 256;   // lanes (threads) per enumeration tile
constexpr uint32_t BOUNDS_MIN_TILES_PER_BLOCK = 8;   // fewer tiles per block of the grid: the search runs without bounds
constexpr int MAXE = MAXT * (MAXT - 1) / 2;   // edges of a task graph without cycles
constexpr uint16_t NOT_HELD = 0xFFFF;
constexpr uint64_t NEED_LIMIT = 1ull << 44;   // micro-requests/s a task may see with per-variant factors
constexpr uint64_t NO_KEY = ~0ull;

// instance flag bits
constexpr uint32_t F_TRUNCATED = 1u;        // cap thinning dropped a choice
constexpr uint32_t F_WIDE      = 2u;        // enumerated with 64-bit keys (32-bit fast path did not fit)
constexpr uint32_t F_OVERFLOW  = 1u << 8;   // replicas, cost or key do not fit
constexpr uint32_t F_EMPTY     = 1u << 9;   // some task has no surviving choice
constexpr uint32_t F_CUT       = 1u << 10;  // bounds on: no candidate fits S_avail, nothing was enumerated
constexpr uint32_t F_MISMATCH  = 1u << 11;  // the enumeration's winner failed the rescoring (internal error)

// One surviving choice of one task at one demand level.
struct __attribute__((aligned(32))) Entry {
    uint32_t lat;     // profiled latency, us
    uint32_t cost;    // replicas * partition units
    double   acc;     // accuracy of its variant
    uint64_t key;     // (cost << idx_bits) | digit * stride   (caller's index order)
    uint32_t rep;     // replicas; mixture mode: m1 | m2 << 16
    uint32_t choice;  // original choice id; mixture mode: c1 | c2 << 16 (c2 = 0xFFFF: one tuple only)
};
static_assert(sizeof(Entry) == 32, "Entry must be 32 bytes");

// Compact stream of the innermost position's entries for the 32-bit fast path: its
// surviving choices grouped by variant, inside a variant in ascending latency (ties:
// ascending digit), each group padded to whole quads with entries that can never
// win (lat = k32 = 0xFFFFFFFF).  One quad is one 64-byte scalar load; the dword
// positions below are used by name in the enumeration kernel's inner loop.
struct XEnt { uint32_t lat; uint32_t k32; };
struct __attribute__((aligned(64))) Quad {
    XEnt     e[4];      // dwords 0-7
    double   acc;       // dwords 8-9: accuracy of the quad's variant
    uint32_t newgrp;    // dword 10: 1 if the accuracy test must be (re)done here: a new
                        //   variant starts, or a tile's range of quads starts
    uint32_t pad[5];
};
static_assert(sizeof(Quad) == 64, "Quad must be 64 bytes");

// Mixture mode: every entry of the innermost position has its own accuracy, so a quad
// holds four (latency, local key, accuracy) triples; the whole stream is in ascending
// latency (ties: ascending digit) and padded with entries that can never win.
struct XEntM { uint32_t lat; uint32_t k32; double acc; };
struct __attribute__((aligned(64))) QuadM { XEntM e[4]; };
static_assert(sizeof(QuadM) == 64, "QuadM must be 64 bytes");
// Single tuples, second copy of the same stream without the headers: four (lat, k32) pairs
// per 32-byte record, read two records deep by the loop that keeps the accuracy outcome per
// variant in scalar registers (it needs neither the accuracy nor the flag).  One record past
// the stream's end is read ahead and never used.
struct __attribute__((aligned(32))) QuadC { XEnt e[4]; };
static_assert(sizeof(QuadC) == 32, "QuadC must be 32 bytes");
// What that loop needs of the digits of the position above the innermost one (position 1): three
// arrays of k_max + 3 words each, one after the other - latencies, 32-bit local keys (four of
// each are read at a time, from any digit), and per digit the first later digit whose variant
// has another accuracy (digits in between share the accuracy outcome of every variant of
// position 0).  A fourth array of the same size holds, per digit of position 2, the first later
// digit of another variant; a fifth and a sixth, per digit of position 1, the smallest local key
// and the lowest latency from that digit to the end of its run (bounds: a run none of whose digits
// can stay within the cost bound or meet the latency SLO is left out as a whole).
constexpr uint32_t ydigit_words(uint32_t k_max) { return k_max + 3; }
constexpr uint32_t YDIGIT_ARRAYS = 6;
// Records of 64 bytes per instance in the stream buffer: k_max Quad (or QuadM), then
// k_max + 1 QuadC, then the arrays of the digits of positions 1 and 2 (YDIGIT_ARRAYS x ydigit_words(k_max) words).
constexpr uint32_t quad_stride(uint32_t k_max)
{
    return k_max + (k_max + 2) / 2 + (YDIGIT_ARRAYS * ydigit_words(k_max) + 15) / 16;
}
constexpr uint32_t quadc_offset(uint32_t k_max) { return k_max; }                          // in Quad units
constexpr uint32_t yrec_offset(uint32_t k_max) { return k_max + (k_max + 2) / 2; }
// Pair stream (single tuples, three in-lane positions): for every digit of position 1 a copy of
// position 0's QuadC records with that digit's local key already added to every key, so that a
// lane's running minimum can stay in one register across all digits of position 1.  Records of
// 32 bytes per instance that are set aside for it (an instance whose stream does not fit runs
// without it), plus one spare record that is read ahead and never used.  Small for many
// instances: all of them together stay below PAIR_BUDGET_BYTES.
constexpr uint32_t PAIR_CAP = 8192;
constexpr uint64_t PAIR_BUDGET_BYTES = 256ull << 20;
constexpr uint32_t pair_records(uint32_t k_max, uint32_t n_inst)
{
    const uint64_t want = (uint64_t)k_max * ((k_max + 3) / 4 + 8);      // every variant pads to whole quads
    const uint64_t share = PAIR_BUDGET_BYTES / 32u / (n_inst ? n_inst : 1u);
    const uint64_t r = want < share ? want : share;
    return r < PAIR_CAP ? (uint32_t)r : PAIR_CAP;
}


// Task graph of one problem, by position.
struct Graph {
    uint32_t T, V, P, B, C;
    uint32_t q;               // queue factor
    uint32_t capacity;        // S_avail, 0 = unlimited
    uint32_t src_mask;        // bit p: position p has no predecessor
    uint32_t sink_mask;       // bit p: position p has no successor
    uint32_t pad0;
    uint8_t  task_at[MAXT];   // task id at position p
    uint8_t  pos_of[MAXT];    // position of task id t
    uint32_t succ[MAXT];      // bit s: position s is a successor of position p (s > p)
    uint32_t mult[MAXT];      // demand multiplier (1/1000ths), by task id
    uint32_t through[MAXT];   // longest path through task t with every other task at
                              // its fastest choice and t itself at zero, by task id
    double   u[MAXT];         // sink share of position p (0 if not a sink)
    double   w[MAXT][MAXT];   // w[p][s] share of p among the predecessors of s (0 if no edge)
    double   amax;            // A_raw with every task on its most accurate variant
    // search-space restrictions of the ablations (Section 4.3, Appendix B), by task id
    uint32_t only_variant[MAXT];   // the only variant allowed, 0xFFFFFFFF = all
    uint32_t only_part;            // the only partition index allowed, 0xFFFFFFFF = all
    uint32_t static_budgets;       // 1: per-task latency and resource budgets apply
    uint32_t lat_ref[MAXT];        // highest latency of the task's reference variant
    uint64_t lat_path[MAXT];       // heaviest path through the task, tasks weighted by lat_ref
    uint32_t unit_budget[MAXT];    // resource share in whole units, 0xFFFFFFFF = none
    // per-variant multiplicative factors (Eq. 4): edges by task id in the caller's order
    uint32_t n_edges;
    uint32_t pad1;
    uint8_t  e_src[MAXE], e_dst[MAXE];
    const uint32_t* fac;      // [n_edges][V] in 1/1000ths, device pointer; null = fixed multipliers
    // tables of this problem, device pointers
    const uint32_t* lat;      // [T][C]
    const uint32_t* thr;      // [T][C]  mrps
    const double*   acc;      // [T][V]
    const uint32_t* units;    // [P]
};

// One search instance: a problem at one demand level.
// Variants of the innermost position whose accuracy masks a wave keeps in scalar registers.
constexpr int MAX_XVAR = 8;

// x / k and x % k for 32-bit x by the reciprocal m = floor(2^32 / k) (k = 1: 2^32 - 1): the
// product's high word is the quotient or one less (x * m / 2^32 lies in (x/k - 1, x/k]), so one
// conditional step finishes it.  The remainder is always below k.
#if defined(__HIPCC__) || defined(__HIP__)
#define JSV_HD __host__ __device__
#else
#define JSV_HD
#endif
JSV_HD inline uint32_t div_by_magic(uint32_t x, uint32_t k, uint32_t m, uint32_t* rem)
{
    uint32_t q = (uint32_t)(((uint64_t)x * m) >> 32);
    uint32_t r = x - q * k;
    if (r >= k) { r -= k; ++q; }
    *rem = r;
    return q;
}
JSV_HD inline uint32_t magic_of(uint32_t k) { return k <= 1u ? 0xFFFFFFFFu : (uint32_t)((1ull << 32) / k); }

struct Instance {
    // inputs (host)
    uint32_t problem;
    uint32_t demand;          // mrps
    uint32_t slo_l;           // us
    uint32_t cap;             // prune cap, 0 = exhaustive
    double   slo_a;           // threshold on A_obj
    double   slo_raw;         // slo_a * amax: threshold on A_raw
    // written by the prune and plan kernels
    uint32_t K[MAXT];         // surviving choices per task id
    uint64_t stride[MAXT];    // prod_{u<t} K_u per task id
    uint64_t space;           // prod K_t
    uint64_t s_out;           // outer combinations = prod of K over positions >= n_in
    uint32_t idx_bits;        // bits of the index part of a key
    uint32_t flags;
    uint32_t n_in;            // positions 0..n_in-1 are looped inside a lane
    uint32_t chunk;           // digits of position n_in-1 per tile
    uint32_t n_chunks;
    uint32_t n_groups;        // ceil(s_out / TILE_LANES)
    uint32_t tiles;           // n_groups * n_chunks
    uint32_t trunc_mask;      // bit t: cap thinning dropped a choice of task id t
    uint64_t tile_begin;      // first global tile of this instance (exclusive scan)
    // 32-bit fast path: inside a lane-tile candidates are compared by
    // (cost of the in-lane positions << lb) | rank, rank = their order by caller index
    uint32_t use32;           // 1 if that fits 31 bits
    uint32_t lb;              // bits of the rank
    uint32_t nq;              // quads in the innermost position's stream
    uint32_t ord[3];          // in-lane positions, least significant caller digit first
    // bounds that let whole lanes and waves sit out (written by the plan kernel)
    uint32_t min_in_cost;     // sum over the in-lane positions of their cheapest entry
    uint32_t min_x_lat;       // lowest latency among the innermost position's entries
    // objective of Eq. 14 (inputs, host): maximise alpha * A_obj - beta * cost
    double   alpha, beta;
    double   alpha_n;         // alpha / A_max: factor on A_raw
    double   inv_beta;        // 1 / beta, or 0 when beta is too small for a cost limit to be derived from an objective
    // per-variant factors (input, host): the one variant task id t is held to in this
    // instance, NOT_HELD = free.  With every task that changes a downstream demand held, the
    // demands of all tasks are fixed and the instance is an ordinary search.
    uint16_t held[MAXT];
    uint32_t min_x_cost;      // cheapest entry of the innermost position (plan kernel)
    uint32_t min_xy_cost;     // plus the cheapest entry of the position above it (if looped in-lane)
    // for the rebalancing of tile sizes once all instances are planned
    uint32_t ko;              // extent of the chunked loop: digits of position n_in-1, or quads of the stream
    uint32_t unit_cost;       // candidates per lane and unit of that loop (clamped)
    uint32_t tile_cost;       // candidates per lane and tile = chunk * unit_cost (clamped)
    uint32_t splittable;      // 1: chunk may still be lowered (not when the stream itself is chunked)
    // the variants of the innermost position in the order of its stream (single tuples): how
    // many, and the accuracy of the first MAX_XVAR of them (plan kernel)
    uint32_t nvx;
    uint32_t pair_nq;         // records per digit of position 1 in the pair stream; 0: no pair stream
    double   xacc[MAX_XVAR];
    uint32_t xqe[MAX_XVAR];   // byte offset in the QuadC copy at which each of them ends (past nvx: the stream's end)
    // floor(2^32 / K[t]) per task id (K = 1: 2^32 - 1), so that the lanes split their combination
    // into digits by a multiplication and one correction instead of a division (plan kernel)
    uint32_t kmagic[MAXT];
    // the same by position instead of task id, with the row of the position's task in the entry
    // table (task id * k_max): the tile set-up reads them with a few wide scalar loads instead of a
    // chain of dependent ones through the task ids (plan kernel)
    uint32_t kpos[MAXT];
    uint32_t mpos[MAXT];
    uint32_t rowpos[MAXT];
    uint32_t sloq;            // floor(slo_l / q): what Eq. 3 leaves for the critical path (plan kernel)
    uint32_t pad_sloq;
};

// Result record as written by the finalize kernel; same layout as jsv_result.
struct ResultRec {
    uint64_t index, full_index, evaluated;
    double   accuracy;
    uint32_t latency_us;
    int32_t  cost_units;
    uint32_t feasible, flags;
    uint16_t choice[MAXT];
    uint32_t replicas[MAXT];
    double   objective;
    uint16_t choice2[MAXT];     // mixture mode: second tuple per task, 0xFFFF = none
    uint32_t replicas2[MAXT];   // mixture mode: its replicas
};

struct SummaryRec {
    int32_t  best_level;
    uint32_t max_demand;
    uint64_t total_tiles;     // written by the scan kernel
    uint32_t done_count;      // finalize blocks finished
    uint32_t any_flags;       // OR of all instance flags
    unsigned long long next_tile;   // work counter of the enumeration kernel: first tile not handed out yet
    uint32_t plan_done;       // plan blocks finished
    uint32_t bounded;         // 1: the enumeration kernel with bounds does the work, 0: the plain one
                              //    (set by the scan: bounds only pay when a block sees many tiles)
    unsigned long long visited;     // entries of the innermost position that waves went through
    uint32_t own_tiles;       // tiles of one run that a block of the enumeration takes by its index
    uint32_t own_rounds;      // rounds of such runs: round r, block b starts at (r * blocks + b) * own_tiles
    uint32_t batch_tiles;     // tiles per ticket of the work counter afterwards; 0: no tickets at all
    uint32_t pad3;
};

// Everything the kernels need to find their data; passed by value.  Every member has a
// default (null / 0 / off), so a Plan that a call site forgets to fill in completely never
// carries a stale mode switch or pointer into a kernel.
struct Plan {
    const Graph* graphs = nullptr;      // [n_problems]
    Instance*    inst = nullptr;        // [n_inst]
    Entry*       entries = nullptr;     // [n_inst][t_max][k_max]   by task id
    uint32_t*    rep = nullptr;         // [n_inst][t_max][c_max]   replicas of every choice
    uint32_t*    cost = nullptr;        // [n_inst][t_max][c_max]
    uint32_t*    k32 = nullptr;         // [n_inst][t_max][k_max]   32-bit local keys (in-lane tasks)
    Quad*        quads = nullptr;       // [n_inst][quad_stride(k_max)]  stream of the innermost position
    QuadC*       pairs = nullptr;       // [n_inst][pair_cap + 1]   pair stream of positions 1 and 0
    uint32_t     pair_cap = 0;          // records of it per instance (0: none)
    uint32_t     pair_pad = 0;          // (explicit, so that the struct has no unnamed padding)
    uint64_t*    partial = nullptr;     // [n_inst][grid]           per-block minima (keys)
    double*      partial_obj = nullptr; // [n_inst][grid]           per-block best objectives (objective mode)
    ResultRec*   results = nullptr;     // [n_inst]
    SummaryRec*  summary = nullptr;
    uint32_t n_inst = 0, t_max = 0, k_max = 0, c_max = 0;
    uint32_t grid = 0;            // blocks of the enumeration kernel
    uint32_t lanes_wanted = 0;    // total lanes the planner tries to expose
    uint32_t objective = 0;       // 0: cheapest feasible; 1: largest alpha*A_obj - beta*cost (Eq. 14)
    uint32_t mix = 0;             // 1: a task may run two tuples side by side (Eq. 2, 6, 7, 9, 10)
    uint32_t bounds = 0;          // 1: skip what latency and capacity bounds exclude; 0: issue every candidate's tests
    uint32_t cut = 0;             // 1: an instance whose cheapest entries together exceed S_avail gets no tiles
    // mixture mode: per (instance, task) a grid of cells (cost 0..S_avail) x (latency class),
    // mix_cells entries each
    uint64_t* cell_acc = nullptr;  // best accuracy seen in the cell (bits of a positive double, 0 = empty)
    uint64_t* cell_id = nullptr;   // lowest option id among those with that accuracy
    uint64_t* cell_pm = nullptr;   // prefix maxima of cell_acc; later reused as a list of kept cells
    uint32_t* cell_list = nullptr; // cells that survive the dominance test
    uint64_t  mix_cells = 0;
    // bounds on: per instance the largest total cost still of interest: S_avail at first, then
    // the cost of the cheapest candidate found so far that meets both SLOs (cost modes only)
    uint32_t* bound = nullptr;     // [n_inst]
    uint64_t* tile_begin = nullptr; // [n_inst] first global tile of every instance, for the search by tile
    // objective mode: per instance the best objective any wave has reached so far, as a 64-bit
    // pattern whose unsigned order is the order of the doubles (so that atomicMax keeps the best)
    unsigned long long* best_obj = nullptr;  // [n_inst]
};

}  // namespace jsv
