// Host side of the C ABI (include/jsv.h): validation, task-graph staging
// (topological order, request shares, A_max, per-task latency slack), device
// memory layout, the launch sequence on the caller's stream, result conversion.
//
// The host does no search arithmetic: replicas, cost, prune, scoring and the
// arg-min all run in the kernels (jsv_kernels.hip).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/jsv.h"
#include "jsv_device.h"
#include "jsv_launch.h"

static_assert(JSV_MAX_TASKS == jsv::MAXT, "header and device limits differ");
static_assert(JSV_MAX_CHOICES == jsv::MAXC, "header and device limits differ");
static_assert(sizeof(jsv_result) == sizeof(jsv::ResultRec), "result layouts differ");

namespace {

using jsv::Graph;
using jsv::Instance;
using jsv::MAXT;

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// One compound system as staged on the host.
struct HostProblem {
    uint32_t T = 0, V = 0, P = 0, B = 0, C = 0;
    std::vector<uint32_t> units, batch, lat, thr;
    std::vector<double> acc;
    bool have_profile = false;
    // graph inputs
    uint32_t E = 0;
    std::vector<uint16_t> src, dst;
    std::vector<uint32_t> mult;
    uint32_t capacity = 0, q = 2;
    bool have_dag = false;
    std::vector<uint32_t> fac;     // [E][V] per-variant factors, empty = fixed multipliers
    // staged
    Graph graph;
    bool staged = false;
};

struct Search {               // per-instance search parameters (batch mode keeps them per problem)
    uint32_t demand = 0, slo_l = 0, cap = 0;
    double slo_a = 0.0;
};

struct Layout {               // offsets into the workspace
    size_t inst, entries, rep, cost, k32, quads, pairs, partial, partial_obj, results, summary, eval, total;
    size_t cell_acc, cell_id, cell_pm, cell_list;     // mixture mode only
    size_t bound, tile_begin, best_obj;
};

}  // namespace

struct jsv_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    int last_hip = 0;
    bool device_ready = false;
    uint32_t grid = 0;                 // upper bound on enumeration blocks (sizes the workspace)
    uint32_t cus = 0;
    // occupancy of the enumeration kernel, remembered for the last table shape
    uint32_t occ_t = 0, occ_k = 0; int occ_obj = -1, occ_blocks = 0;      // occ_obj: kernel mode

    HostProblem single;
    std::vector<HostProblem> batch;
    std::vector<Search> batch_search;
    bool batch_mode = false;
    bool dirty = true;                 // host problems changed since the last upload
    bool space_a = true, space_s = true, space_t = true;   // ablation switches
    bool mix = false;                  // mixtures of two tuples per task
    bool bounds = true;                // skip lanes and waves that latency / capacity bounds exclude
    int geo_blocks = 0;                // launch geometry overrides (jsv_set_geometry), 0 = automatic
    int geo_lanes_percent = 0;
    int objective = 0;                 // Eq. 14 mode and weights
    double alpha = 1.0, beta = 0.035;

    void* d_problems = nullptr;        // graphs + tables
    size_t d_problems_bytes = 0;
    uint32_t n_problems = 0;

    void* ws_own = nullptr;  size_t ws_own_bytes = 0;
    void* ws_lent = nullptr; size_t ws_lent_bytes = 0;

    void* pinned = nullptr;  size_t pinned_bytes = 0;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};

    // graph mode: the copy-kernels-copy sequence of a search, captured once per shape
    bool graph_mode = false;
    hipGraph_t graph = nullptr;
    hipGraphExec_t graph_exec = nullptr;
    jsv::Plan graph_plan;              // what the captured sequence was built for
    const void* graph_pin = nullptr;
};

namespace {

#define HIP_TRY(ctx, expr)                                     \
    do {                                                       \
        hipError_t e_ = (expr);                                \
        if (e_ != hipSuccess) { (ctx)->last_hip = (int)e_; return JSV_E_DEVICE; } \
    } while (0)

// ---- memory for callers that cannot allocate ---------------------------------------------
// jsv_search_static keeps everything a search needs on the device - the problem blob at the
// front, the workspace behind it - in this array instead of allocated memory.  One copy per
// GPU, held until the process ends, shared by every context on that GPU; it keeps the last
// call's contents (the blob and the instance records are rewritten by every call, counters and
// partial results are reset by the kernels themselves).  In host code the array's name is only a
// handle for hipGetSymbolAddress: the device address it yields, per device, is what kernels
// and copies get.
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[JSV_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
unsigned char* g_scratch_ptr[MAX_DEVICES];      // device address of `scratch` on each GPU, null = not asked yet
std::mutex g_scratch_mutex;

struct StaticArena {        // a search that lives in the static array
    unsigned char* base;    // its device address on the context's GPU
    size_t blob_bytes;      // the problem blob takes this much of its front (256-byte multiple)
};

// Device address of the static array on the context's GPU, which must be current.
int static_scratch(jsv_ctx* ctx, unsigned char** out)
{
    if (ctx->device < 0 || ctx->device >= MAX_DEVICES) return JSV_E_BADARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[ctx->device]) {
        void* p = nullptr;
        HIP_TRY(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return JSV_E_DEVICE;
        g_scratch_ptr[ctx->device] = (unsigned char*)p;
    }
    *out = g_scratch_ptr[ctx->device];
    return JSV_OK;
}

int check_profile(uint32_t T, uint32_t V, uint32_t P, uint32_t B, const uint32_t* units,
                  const uint32_t* batch, const uint32_t* lat, const uint32_t* thr, const double* acc,
                  HostProblem& hp)
{
    if (!units || !batch || !lat || !acc) return JSV_E_NULL;
    if (T == 0 || T > JSV_MAX_TASKS || V == 0 || P == 0 || B == 0) return JSV_E_BADARG;
    const uint64_t C64 = (uint64_t)V * P * B;
    if (C64 > JSV_MAX_CHOICES) return JSV_E_BADARG;
    const uint32_t C = (uint32_t)C64;
    for (uint32_t p = 0; p < P; ++p) if (units[p] == 0) return JSV_E_BADARG;
    for (uint32_t b = 0; b < B; ++b) if (batch[b] == 0) return JSV_E_BADARG;
    const size_t n = (size_t)T * C;
    std::vector<uint32_t> h(n);
    for (size_t k = 0; k < n; ++k) {
        if (lat[k] == 0) return JSV_E_BADARG;
        if (thr) {
            if (thr[k] == 0) return JSV_E_BADARG;
            h[k] = thr[k];
        } else {
            // one batch of batch[b] requests every latency microseconds, in milli-requests/s
            const uint64_t v = (uint64_t)batch[k % B] * 1000000000ull / lat[k];
            if (v > 0xFFFFFFFFull) return JSV_E_OVERFLOW;
            if (v == 0) return JSV_E_BADARG;
            h[k] = (uint32_t)v;
        }
    }
    for (size_t k = 0; k < (size_t)T * V; ++k)
        if (!(acc[k] > 0.0 && acc[k] <= 1.0)) return JSV_E_BADARG;
    hp.T = T; hp.V = V; hp.P = P; hp.B = B; hp.C = C;
    hp.units.assign(units, units + P);
    hp.batch.assign(batch, batch + B);
    hp.lat.assign(lat, lat + n);
    hp.thr.swap(h);
    hp.acc.assign(acc, acc + (size_t)T * V);
    hp.fac.clear();
    hp.have_profile = true;
    hp.staged = false;
    return JSV_OK;
}

int check_dag(uint32_t T, uint32_t E, const uint16_t* src, const uint16_t* dst, const uint32_t* mult,
              uint32_t capacity, uint32_t q, HostProblem& hp)
{
    if (!mult || (E && (!src || !dst))) return JSV_E_NULL;
    if (T == 0 || T > JSV_MAX_TASKS || q == 0) return JSV_E_BADARG;
    bool adj[MAXT][MAXT] = {};
    for (uint32_t e = 0; e < E; ++e) {
        const uint32_t a = src[e], b = dst[e];
        if (a >= T || b >= T || a == b || adj[a][b]) return JSV_E_BADARG;
        adj[a][b] = true;
    }
    for (uint32_t t = 0; t < T; ++t) if (mult[t] == 0) return JSV_E_BADARG;
    // cycle check (Kahn): strip tasks without remaining predecessors
    {
        int indeg[MAXT] = {};
        bool gone[MAXT] = {};
        for (uint32_t a = 0; a < T; ++a) for (uint32_t b = 0; b < T; ++b) indeg[b] += adj[a][b];
        for (uint32_t round = 0; round < T; ++round) {
            int pick = -1;
            for (uint32_t t = 0; t < T; ++t) if (!gone[t] && indeg[t] == 0) { pick = (int)t; break; }
            if (pick < 0) return JSV_E_CYCLE;
            gone[pick] = true;
            for (uint32_t b = 0; b < T; ++b) if (adj[pick][b]) --indeg[b];
        }
    }
    hp.E = E;
    hp.src.assign(src, src + E);
    hp.dst.assign(dst, dst + E);
    hp.mult.assign(mult, mult + T);
    hp.capacity = capacity; hp.q = q;
    hp.have_dag = true;
    hp.staged = false;
    hp.fac.clear();                // factors belong to the edge list they were given for
    if (!hp.have_profile) hp.T = T;
    return JSV_OK;
}

struct SpaceFlags { bool a = true, s = true, t = true; };

// Topological order, shares, A_max, per-task slack, search-space restrictions: fills hp.graph
// (device pointers left null).
int stage_graph(HostProblem& hp, const SpaceFlags& sp = SpaceFlags())
{
    const uint32_t T = hp.T, C = hp.C, V = hp.V;
    Graph& g = hp.graph;
    std::memset(&g, 0, sizeof g);
    g.T = T; g.V = V; g.P = hp.P; g.B = hp.B; g.C = C; g.q = hp.q; g.capacity = hp.capacity;
    bool adj[MAXT][MAXT] = {};
    for (uint32_t e = 0; e < hp.E; ++e) adj[hp.src[e]][hp.dst[e]] = true;
    g.n_edges = hp.E;              // at most MAXE: no repeated edge, no cycle
    for (uint32_t e = 0; e < hp.E; ++e) { g.e_src[e] = (uint8_t)hp.src[e]; g.e_dst[e] = (uint8_t)hp.dst[e]; }
    // Kahn, lowest task id first
    {
        int indeg[MAXT] = {};
        bool gone[MAXT] = {};
        for (uint32_t a = 0; a < T; ++a) for (uint32_t b = 0; b < T; ++b) indeg[b] += adj[a][b];
        for (uint32_t p = 0; p < T; ++p) {
            int pick = -1;
            for (uint32_t t = 0; t < T; ++t) if (!gone[t] && indeg[t] == 0) { pick = (int)t; break; }
            if (pick < 0) return JSV_E_CYCLE;
            gone[pick] = true;
            g.task_at[p] = (uint8_t)pick;
            g.pos_of[pick] = (uint8_t)p;
            for (uint32_t b = 0; b < T; ++b) if (adj[pick][b]) --indeg[b];
        }
    }
    uint64_t sink_total = 0;
    for (uint32_t t = 0; t < T; ++t) {
        bool has_succ = false, has_pred = false;
        for (uint32_t o = 0; o < T; ++o) { has_succ |= adj[t][o]; has_pred |= adj[o][t]; }
        const uint32_t p = g.pos_of[t];
        if (!has_succ) { g.sink_mask |= 1u << p; sink_total += hp.mult[t]; }
        if (!has_pred) g.src_mask |= 1u << p;
        g.mult[t] = hp.mult[t];
    }
    for (uint32_t s = 0; s < T; ++s) {            // s: head of the edges
        uint64_t in_total = 0;
        for (uint32_t a = 0; a < T; ++a) if (adj[a][s]) in_total += hp.mult[a];
        for (uint32_t a = 0; a < T; ++a) {
            if (!adj[a][s]) continue;
            const uint32_t pa = g.pos_of[a], ps = g.pos_of[s];
            g.succ[pa] |= 1u << ps;
            g.w[pa][ps] = (double)hp.mult[a] / (double)in_total;
        }
        if ((g.sink_mask >> g.pos_of[s]) & 1u) g.u[g.pos_of[s]] = (double)hp.mult[s] / (double)sink_total;
    }
    // A_max: the backward recursion with every task on its most accurate variant, in the one
    // order of operations that the kernels use for every candidate (see jsv_device.h): successors
    // added by fma in descending position, sources added in descending position, position 0 joined
    // by one fma.  The all-best assignment then reproduces A_max bit for bit on the device, so a
    // threshold of exactly 1.0 accepts it.
    {
#pragma clang fp contract(off)
        double H[MAXT] = {};
        double raw = 0.0;
        for (int p = (int)T - 1; p >= 0; --p) {
            const uint32_t t = g.task_at[p];
            double a = hp.acc[(size_t)t * V];
            for (uint32_t v = 1; v < V; ++v) a = std::max(a, hp.acc[(size_t)t * V + v]);
            double hs = 0.0;
            for (int s = (int)T - 1; s > p; --s) if ((g.succ[p] >> s) & 1u) hs = std::fma(g.w[p][s], H[s], hs);
            const double inner = ((g.sink_mask >> p) & 1u) ? g.u[p] : hs;
            if (p == 0) { raw = std::fma(a, inner, raw); break; }      // position 0 is always a source
            const double prod = a * inner;
            H[p] = prod;
            if ((g.src_mask >> p) & 1u) { const double sum = raw + prod; raw = sum; }
        }
        g.amax = raw;
    }
    // Latency range and, per task, the longest path through it with every other task at its
    // fastest choice (used by the prune's latency filter).
    uint64_t lo[MAXT], hi_sum = 0;
    for (uint32_t t = 0; t < T; ++t) {
        uint32_t mn = hp.lat[(size_t)t * C], mx = mn;
        for (uint32_t c = 1; c < C; ++c) { mn = std::min(mn, hp.lat[(size_t)t * C + c]); mx = std::max(mx, hp.lat[(size_t)t * C + c]); }
        lo[t] = mn; hi_sum += mx;
    }
    if ((uint64_t)hp.q * hi_sum > 0xFFFFFFFFull) return JSV_E_OVERFLOW;
    uint64_t up[MAXT] = {}, down[MAXT] = {};
    for (uint32_t p = 0; p < T; ++p)
        for (uint32_t s = p + 1; s < T; ++s)
            if ((g.succ[p] >> s) & 1u) up[s] = std::max(up[s], up[p] + lo[g.task_at[p]]);
    for (int p = (int)T - 1; p >= 0; --p)
        for (uint32_t s = p + 1; s < T; ++s)
            if ((g.succ[p] >> s) & 1u) down[p] = std::max(down[p], down[s] + lo[g.task_at[s]]);
    for (uint32_t p = 0; p < T; ++p) g.through[g.task_at[p]] = (uint32_t)(up[p] + down[p]);

    // Restrictions of the ablations.  Reference tuple of a task: its most accurate variant
    // (lowest id among equals) over the allowed partitions and all batches.
    uint32_t whole = 0;
    for (uint32_t p = 1; p < hp.P; ++p) if (hp.units[p] > hp.units[whole]) whole = p;
    g.only_part = sp.s ? 0xFFFFFFFFu : whole;
    g.static_budgets = sp.t ? 0u : 1u;
    double need[MAXT], need_total = 0.0;
    for (uint32_t t = 0; t < T; ++t) {
        uint32_t bv = 0;
        for (uint32_t v = 1; v < V; ++v) if (hp.acc[(size_t)t * V + v] > hp.acc[(size_t)t * V + bv]) bv = v;
        g.only_variant[t] = sp.a ? 0xFFFFFFFFu : bv;
        uint32_t lmax = 0, best_thr = 0, best_units = 0;
        for (uint32_t p = 0; p < hp.P; ++p) {
            if (!sp.s && p != whole) continue;
            for (uint32_t b = 0; b < hp.B; ++b) {
                const size_t k = (size_t)t * C + ((size_t)bv * hp.P + p) * hp.B + b;
                lmax = std::max(lmax, hp.lat[k]);
                if (hp.thr[k] > best_thr) { best_thr = hp.thr[k]; best_units = hp.units[p]; }
            }
        }
        g.lat_ref[t] = lmax;
        need[t] = ((double)hp.mult[t] * (double)best_units) / (double)best_thr;
        need_total += need[t];
    }
    {   // heaviest path through each task with the tasks weighted by their reference latency
        uint64_t upw[MAXT] = {}, downw[MAXT] = {};
        for (uint32_t p = 0; p < T; ++p)
            for (uint32_t s = p + 1; s < T; ++s)
                if ((g.succ[p] >> s) & 1u) upw[s] = std::max(upw[s], upw[p] + g.lat_ref[g.task_at[p]]);
        for (int p = (int)T - 1; p >= 0; --p)
            for (uint32_t s = p + 1; s < T; ++s)
                if ((g.succ[p] >> s) & 1u) downw[p] = std::max(downw[p], downw[s] + g.lat_ref[g.task_at[s]]);
        for (uint32_t p = 0; p < T; ++p) {
            const uint32_t t = g.task_at[p];
            g.lat_path[t] = upw[p] + g.lat_ref[t] + downw[p];
        }
    }
    for (uint32_t t = 0; t < T; ++t) {
        g.unit_budget[t] = 0xFFFFFFFFu;
        if (!sp.t && hp.capacity != 0) {
            const double share = std::floor((double)hp.capacity * (need[t] / need_total));
            g.unit_budget[t] = share >= 4294967295.0 ? 0xFFFFFFFEu : (uint32_t)share;
        }
    }
    hp.staged = true;
    return JSV_OK;
}

int ensure_device(jsv_ctx* ctx)
{
    if (ctx->device_ready) { HIP_TRY(ctx, hipSetDevice(ctx->device)); return JSV_OK; }
    HIP_TRY(ctx, hipSetDevice(ctx->device));
    int cus = 0;
    HIP_TRY(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device));
    if (cus <= 0) cus = 256;
    ctx->cus = (uint32_t)cus;
    ctx->grid = (uint32_t)cus * 8u;
    ctx->device_ready = true;
    return JSV_OK;
}

int ensure_events(jsv_ctx* ctx)
{
    for (auto& e : ctx->ev) if (!e) HIP_TRY(ctx, hipEventCreate(&e));
    return JSV_OK;
}

void drop_graph(jsv_ctx* ctx)
{
    if (ctx->graph_exec) { (void)hipGraphExecDestroy(ctx->graph_exec); ctx->graph_exec = nullptr; }
    if (ctx->graph) { (void)hipGraphDestroy(ctx->graph); ctx->graph = nullptr; }
    ctx->graph_pin = nullptr;
}

int ensure_pinned(jsv_ctx* ctx, size_t bytes)
{
    if (ctx->pinned_bytes >= bytes) return JSV_OK;
    if (ctx->pinned) { HIP_TRY(ctx, hipHostFree(ctx->pinned)); ctx->pinned = nullptr; ctx->pinned_bytes = 0; }
    const size_t want = std::max(bytes, (size_t)1 << 16);
    HIP_TRY(ctx, hipHostMalloc(&ctx->pinned, want, hipHostMallocDefault));
    ctx->pinned_bytes = want;
    return JSV_OK;
}

// Graphs and tables of `n` problems as one blob that will live at device address `base`
// (graph pointers are device addresses inside it).  base = nullptr only sizes the blob.
size_t build_blob(const HostProblem* hps, uint32_t n, const unsigned char* base, std::vector<unsigned char>* blob)
{
    size_t off = align_up(sizeof(Graph) * n);
    std::vector<size_t> o_lat(n), o_thr(n), o_acc(n), o_units(n), o_fac(n);
    for (uint32_t k = 0; k < n; ++k) {
        const HostProblem& hp = hps[k];
        o_acc[k] = off;   off = align_up(off + hp.acc.size() * sizeof(double));
        o_lat[k] = off;   off = align_up(off + hp.lat.size() * sizeof(uint32_t));
        o_thr[k] = off;   off = align_up(off + hp.thr.size() * sizeof(uint32_t));
        o_units[k] = off; off = align_up(off + hp.units.size() * sizeof(uint32_t));
        o_fac[k] = off;   off = align_up(off + hp.fac.size() * sizeof(uint32_t));
    }
    if (!blob) return off;
    blob->assign(off, 0);
    for (uint32_t k = 0; k < n; ++k) {
        const HostProblem& hp = hps[k];
        Graph g = hp.graph;
        g.acc = (const double*)(base + o_acc[k]);
        g.lat = (const uint32_t*)(base + o_lat[k]);
        g.thr = (const uint32_t*)(base + o_thr[k]);
        g.units = (const uint32_t*)(base + o_units[k]);
        g.fac = hp.fac.empty() ? nullptr : (const uint32_t*)(base + o_fac[k]);
        std::memcpy(blob->data() + sizeof(Graph) * k, &g, sizeof g);
        std::memcpy(blob->data() + o_acc[k], hp.acc.data(), hp.acc.size() * sizeof(double));
        std::memcpy(blob->data() + o_lat[k], hp.lat.data(), hp.lat.size() * sizeof(uint32_t));
        std::memcpy(blob->data() + o_thr[k], hp.thr.data(), hp.thr.size() * sizeof(uint32_t));
        std::memcpy(blob->data() + o_units[k], hp.units.data(), hp.units.size() * sizeof(uint32_t));
        if (!hp.fac.empty()) std::memcpy(blob->data() + o_fac[k], hp.fac.data(), hp.fac.size() * sizeof(uint32_t));
    }
    return off;
}

// Upload the blob of `n` problems into library-owned device memory (grow-only).
int upload_problems(jsv_ctx* ctx, HostProblem* hps, uint32_t n)
{
    const size_t bytes = build_blob(hps, n, nullptr, nullptr);
    if (ctx->d_problems_bytes < bytes) {
        if (ctx->d_problems) { HIP_TRY(ctx, hipFree(ctx->d_problems)); ctx->d_problems = nullptr; ctx->d_problems_bytes = 0; }
        HIP_TRY(ctx, hipMalloc(&ctx->d_problems, bytes));
        ctx->d_problems_bytes = bytes;
    }
    std::vector<unsigned char> blob;
    build_blob(hps, n, (const unsigned char*)ctx->d_problems, &blob);
    HIP_TRY(ctx, hipMemcpyAsync(ctx->d_problems, blob.data(), bytes, hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));      // blob is a local buffer
    ctx->n_problems = n;
    ctx->dirty = false;
    return JSV_OK;
}

Layout make_layout(uint32_t n_inst, uint32_t t_max, uint32_t k_max, uint32_t c_max, uint32_t grid,
                   uint32_t n_eval, uint64_t mix_cells = 0)
{
    Layout L;
    size_t off = 0;
    L.inst = off;    off = align_up(off + sizeof(Instance) * n_inst);
    L.entries = off; off = align_up(off + sizeof(jsv::Entry) * (size_t)n_inst * t_max * k_max);
    L.rep = off;     off = align_up(off + sizeof(uint32_t) * (size_t)n_inst * t_max * c_max);
    L.cost = off;    off = align_up(off + sizeof(uint32_t) * (size_t)n_inst * t_max * c_max);
    L.k32 = off;     off = align_up(off + sizeof(uint32_t) * (size_t)n_inst * t_max * k_max);
    L.quads = off;   off = align_up(off + sizeof(jsv::Quad) * (size_t)n_inst * jsv::quad_stride(k_max));
    L.pairs = off;   off = align_up(off + sizeof(jsv::QuadC) * (size_t)n_inst * (jsv::pair_records(k_max, n_inst) + 1));
    L.partial = off; off = align_up(off + sizeof(uint64_t) * (size_t)n_inst * grid);
    L.partial_obj = off; off = align_up(off + sizeof(double) * (size_t)n_inst * grid);
    L.results = off; off = align_up(off + sizeof(jsv::ResultRec) * n_inst);
    L.summary = off; off = align_up(off + sizeof(jsv::SummaryRec));
    L.bound = off;   off = align_up(off + sizeof(uint32_t) * n_inst);
    L.tile_begin = off; off = align_up(off + sizeof(uint64_t) * n_inst);
    L.best_obj = off; off = align_up(off + sizeof(uint64_t) * n_inst);
    L.eval = off;    // index u64, latency u32, replicas u32*T, cost i32, accuracy f64, mask u8, bad u32
    off = align_up(off + (size_t)n_eval * (8 + 4 + 4 * MAXT + 4 + 8 + 1) + 6 * ALIGN);
    const size_t blocks = (size_t)n_inst * t_max;
    L.cell_acc = off;  off = align_up(off + sizeof(uint64_t) * blocks * mix_cells);
    L.cell_id = off;   off = align_up(off + sizeof(uint64_t) * blocks * mix_cells);
    L.cell_pm = off;   off = align_up(off + sizeof(uint64_t) * blocks * mix_cells);
    L.cell_list = off; off = align_up(off + sizeof(uint32_t) * blocks * mix_cells);
    L.total = off;
    return L;
}

int get_workspace(jsv_ctx* ctx, size_t bytes, unsigned char** out)
{
    if (ctx->ws_lent) {
        if (ctx->ws_lent_bytes < bytes) return JSV_E_WORKSPACE;
        *out = (unsigned char*)ctx->ws_lent;
        return JSV_OK;
    }
    if (ctx->ws_own_bytes < bytes) {
        if (ctx->ws_own) { HIP_TRY(ctx, hipFree(ctx->ws_own)); ctx->ws_own = nullptr; ctx->ws_own_bytes = 0; }
        HIP_TRY(ctx, hipMalloc(&ctx->ws_own, bytes));
        ctx->ws_own_bytes = bytes;
    }
    *out = (unsigned char*)ctx->ws_own;
    return JSV_OK;
}

uint32_t k_max_of(const HostProblem& hp, uint32_t cap) { return cap ? std::min(cap, hp.C) : hp.C; }

// The one place a Plan is built: all bytes zero (padding too: graph mode compares plans with
// memcmp), every buffer pointer from the layout, every mode switch off unless the context has it
// on.  Callers set what is theirs alone afterwards (grid, lanes_wanted).
jsv::Plan make_plan(const jsv_ctx* ctx, const void* graphs, const Layout& L, unsigned char* ws, uint32_t n_inst,
                    uint32_t t_max, uint32_t k_max, uint32_t c_max, uint64_t mix_cells)
{
    jsv::Plan pl;
    std::memset((void*)&pl, 0, sizeof pl);
    pl.graphs = (const Graph*)graphs;
    pl.inst = (Instance*)(ws + L.inst);
    pl.entries = (jsv::Entry*)(ws + L.entries);
    pl.rep = (uint32_t*)(ws + L.rep);
    pl.cost = (uint32_t*)(ws + L.cost);
    pl.k32 = (uint32_t*)(ws + L.k32);
    pl.quads = (jsv::Quad*)(ws + L.quads);
    pl.pairs = (jsv::QuadC*)(ws + L.pairs);
    pl.pair_cap = jsv::pair_records(k_max, n_inst);
    pl.partial = (uint64_t*)(ws + L.partial);
    pl.partial_obj = (double*)(ws + L.partial_obj);
    pl.results = (jsv::ResultRec*)(ws + L.results);
    pl.summary = (jsv::SummaryRec*)(ws + L.summary);
    pl.bound = (uint32_t*)(ws + L.bound);
    pl.tile_begin = (uint64_t*)(ws + L.tile_begin);
    pl.best_obj = (unsigned long long*)(ws + L.best_obj);
    pl.n_inst = n_inst; pl.t_max = t_max; pl.k_max = k_max; pl.c_max = c_max;
    pl.objective = (uint32_t)ctx->objective;
    if (mix_cells != 0) {
        pl.mix = 1u;
        pl.mix_cells = mix_cells;
        pl.cell_acc = (uint64_t*)(ws + L.cell_acc);
        pl.cell_id = (uint64_t*)(ws + L.cell_id);
        pl.cell_pm = (uint64_t*)(ws + L.cell_pm);
        pl.cell_list = (uint32_t*)(ws + L.cell_list);
    }
    return pl;
}

int check_search_args(const HostProblem& hp, uint32_t demand, double slo_a, uint32_t cap)
{
    if (demand == 0) return JSV_E_BADARG;
    if (!(slo_a == slo_a)) return JSV_E_BADARG;                  // NaN
    if (cap != 0 && cap < 2 * hp.V) return JSV_E_BADARG;
    return JSV_OK;
}

// The whole device pass for n_inst instances whose parameters are in `inst` (host copies).
// With `sa` the search lives in the static array: no allocation of any kind, instance records
// copied straight from `inst` and results straight into `out`, no events (no timing).
int run_search(jsv_ctx* ctx, std::vector<Instance>& inst, uint32_t t_max, uint32_t k_max, uint32_t c_max,
               jsv_result* out, jsv_summary* summary, uint64_t mix_cells = 0, const StaticArena* sa = nullptr)
{
    const uint32_t n = (uint32_t)inst.size();
    if (jsv::enumerate_lds_bytes(t_max, k_max) > 128 * 1024 || jsv::prune_lds_bytes(c_max) > 64 * 1024)
        return JSV_E_BADARG;
    if (mix_cells != 0 && jsv::mix_lds_bytes(c_max) > 64 * 1024) return JSV_E_BADARG;
    const Layout L = make_layout(n, t_max, k_max, c_max, ctx->grid, 0, mix_cells);
    unsigned char* ws = nullptr;
    const void* graphs = ctx->d_problems;
    const size_t in_bytes = sizeof(Instance) * n;
    // result records and the summary are neighbours in the workspace: one copy brings both
    const size_t res_bytes = L.summary - L.results;             // the records, padded to the summary's offset
    const size_t out_bytes = res_bytes + sizeof(jsv::SummaryRec);
    unsigned char* pin_in = (unsigned char*)inst.data();
    unsigned char* pin_out = nullptr;
    int rc = JSV_OK;
    if (sa) {
        if (sa->blob_bytes + L.total > JSV_STATIC_SCRATCH_BYTES || ctx->graph_mode) return JSV_E_WORKSPACE;
        ws = sa->base + sa->blob_bytes;
        graphs = sa->base;
    } else {
        rc = get_workspace(ctx, L.total, &ws);
        if (rc) return rc;
        rc = ensure_pinned(ctx, align_up(in_bytes) + out_bytes);
        if (rc) return rc;
        rc = ensure_events(ctx);
        if (rc) return rc;
        pin_in = (unsigned char*)ctx->pinned;
        pin_out = pin_in + align_up(in_bytes);
        std::memcpy(pin_in, inst.data(), in_bytes);
    }

    jsv::Plan pl = make_plan(ctx, graphs, L, ws, n, t_max, k_max, c_max, mix_cells);
    // Bounds pay only when a block sees many tiles (the device decides that from the real tile
    // count).  Where even an upper estimate of the tiles - every list full, 64 candidates per
    // lane and tile - stays below that, the variant with bounds is not launched at all.  Instances
    // that no candidate can fit are still dropped at plan time (cut).
    bool with_bounds = ctx->bounds;
    if (with_bounds) {
        double most = 0.0;
        for (uint32_t k = 0; k < n; ++k) {
            const HostProblem& hp = ctx->batch_mode ? ctx->batch[inst[k].problem] : ctx->single;
            const double kk = mix_cells ? (double)k_max : (double)k_max_of(hp, inst[k].cap);
            most += std::pow(kk, (double)hp.T) / (64.0 * jsv::TILE_LANES) + 1.0;
        }
        if (most < (double)ctx->grid * (double)jsv::BOUNDS_MIN_TILES_PER_BLOCK) with_bounds = false;
    }
    pl.bounds = with_bounds ? 1u : 0u;
    pl.cut = ctx->bounds ? 1u : 0u;
    const int mode = jsv::enumerate_mode(ctx->objective != 0, pl.mix != 0) * 2 + (with_bounds ? 1 : 0);
    if (ctx->occ_t != t_max || ctx->occ_k != k_max || ctx->occ_obj != mode) {
        int blocks = 0;
        HIP_TRY(ctx, jsv::enumerate_blocks_per_cu(t_max, k_max, mode / 2, with_bounds, &blocks));
        ctx->occ_t = t_max; ctx->occ_k = k_max; ctx->occ_obj = mode; ctx->occ_blocks = blocks;
    }
    const int per_cu = ctx->occ_blocks;
    if (per_cu < 1) return JSV_E_BADARG;
    int blocks = std::min(per_cu, 8);                        // everything launched is resident
    if (ctx->geo_blocks > 0) blocks = std::min(blocks, ctx->geo_blocks);
    pl.grid = ctx->cus * (uint32_t)blocks;
    // lanes the planner tries to keep busy per instance: all that can be resident, shared evenly
    uint64_t lanes = (uint64_t)ctx->grid * jsv::TILE_LANES / n;
    if (ctx->geo_lanes_percent > 0) lanes = lanes * (uint64_t)ctx->geo_lanes_percent / 100u;
    pl.lanes_wanted = (uint32_t)std::max<uint64_t>(64, std::min<uint64_t>(lanes, 0x7FFFFFFF));

    hipStream_t st = ctx->stream;
    bool timed_kernels = true;
    jsv::SummaryRec sr;
    std::memset(&sr, 0, sizeof sr);
    if (ctx->graph_mode && !sa) {
        // Replay the captured sequence when nothing it was built from has changed: same
        // buffers, shapes, grid and objective (the instance records travel through the pinned
        // buffer, so new demands and SLOs need no new capture).
        if (!ctx->graph_exec || std::memcmp(&ctx->graph_plan, &pl, sizeof pl) != 0 || ctx->graph_pin != pin_in) {
            drop_graph(ctx);
            HIP_TRY(ctx, hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
            hipError_t e = hipMemcpyAsync(pl.inst, pin_in, in_bytes, hipMemcpyHostToDevice, st);
            if (e == hipSuccess) e = jsv::launch_prune_plan_scan(pl, st);
            if (e == hipSuccess) e = jsv::launch_enumerate(pl, st);
            if (e == hipSuccess) e = jsv::launch_finalize(pl, st);
            if (e == hipSuccess) e = hipMemcpyAsync(pin_out, pl.results, out_bytes, hipMemcpyDeviceToHost, st);
            hipGraph_t g = nullptr;
            const hipError_t e2 = hipStreamEndCapture(st, &g);       // always leave capture mode
            if (e != hipSuccess || e2 != hipSuccess) {
                if (g) (void)hipGraphDestroy(g);
                ctx->last_hip = (int)(e != hipSuccess ? e : e2);
                return JSV_E_DEVICE;
            }
            ctx->graph = g;
            HIP_TRY(ctx, hipGraphInstantiate(&ctx->graph_exec, ctx->graph, nullptr, nullptr, 0));
            std::memcpy((void*)&ctx->graph_plan, &pl, sizeof pl);
            ctx->graph_pin = pin_in;
        }
        HIP_TRY(ctx, hipEventRecord(ctx->ev[0], st));
        HIP_TRY(ctx, hipGraphLaunch(ctx->graph_exec, st));
        HIP_TRY(ctx, hipEventRecord(ctx->ev[3], st));
        timed_kernels = false;
    } else if (sa) {
        timed_kernels = false;
        HIP_TRY(ctx, hipMemcpyAsync(pl.inst, pin_in, in_bytes, hipMemcpyHostToDevice, st));
        HIP_TRY(ctx, jsv::launch_prune_plan_scan(pl, st));
        HIP_TRY(ctx, jsv::launch_enumerate(pl, st));
        HIP_TRY(ctx, jsv::launch_finalize(pl, st));
        HIP_TRY(ctx, hipMemcpyAsync(out, pl.results, sizeof(jsv::ResultRec) * n, hipMemcpyDeviceToHost, st));
        HIP_TRY(ctx, hipMemcpyAsync(&sr, pl.summary, sizeof(jsv::SummaryRec), hipMemcpyDeviceToHost, st));
    } else {
        HIP_TRY(ctx, hipMemcpyAsync(pl.inst, pin_in, in_bytes, hipMemcpyHostToDevice, st));
        HIP_TRY(ctx, hipEventRecord(ctx->ev[0], st));
        HIP_TRY(ctx, jsv::launch_prune_plan_scan(pl, st));
        HIP_TRY(ctx, hipEventRecord(ctx->ev[1], st));
        HIP_TRY(ctx, jsv::launch_enumerate(pl, st));
        HIP_TRY(ctx, hipEventRecord(ctx->ev[2], st));
        HIP_TRY(ctx, jsv::launch_finalize(pl, st));
        HIP_TRY(ctx, hipEventRecord(ctx->ev[3], st));
        HIP_TRY(ctx, hipMemcpyAsync(pin_out, pl.results, out_bytes, hipMemcpyDeviceToHost, st));
    }
    HIP_TRY(ctx, hipStreamSynchronize(st));

    if (!sa) std::memcpy(&sr, pin_out + res_bytes, sizeof sr);
    if (sr.any_flags & jsv::F_OVERFLOW) return JSV_E_OVERFLOW;
    if (sr.any_flags & jsv::F_MISMATCH) return JSV_E_INTERNAL;
    if (!sa) std::memcpy(out, pin_out, sizeof(jsv::ResultRec) * n);
    uint64_t enumerated = 0;                        // candidates of the instances that were enumerated at all
    for (uint32_t k = 0; k < n; ++k) {
        if (!(out[k].flags & jsv::F_CUT)) enumerated += out[k].evaluated;
        out[k].flags &= (jsv::F_TRUNCATED | jsv::F_WIDE);
    }
    if (summary) {
        float ms_all = 0.f, ms_enum = 0.f;
        if (!sa) HIP_TRY(ctx, hipEventElapsedTime(&ms_all, ctx->ev[0], ctx->ev[3]));
        if (timed_kernels) HIP_TRY(ctx, hipEventElapsedTime(&ms_enum, ctx->ev[1], ctx->ev[2]));
        summary->best_level = sr.best_level;
        summary->max_demand_mrps = sr.max_demand;
        summary->seconds_device = ms_all * 1e-3;
        summary->seconds_enumerate = ms_enum * 1e-3;
        if ((with_bounds && sr.bounded) || ctx->mix) summary->candidates_visited = (uint64_t)sr.visited * 64u;
        else summary->candidates_visited = enumerated;     // the plain kernel issues every candidate's tests
    }
    return JSV_OK;
}

Instance make_instance(const jsv_ctx* ctx, const HostProblem& hp, uint32_t problem, const Search& s)
{
    Instance in;
    std::memset(&in, 0, sizeof in);
    in.alpha = ctx->alpha; in.beta = ctx->beta;
    in.alpha_n = ctx->alpha / hp.graph.amax;
    in.inv_beta = ctx->beta > 1e-9 * (ctx->alpha + 1.0) ? 1.0 / ctx->beta : 0.0;    // (else rounding could reach a unit of cost)
    in.problem = problem;
    in.demand = s.demand; in.slo_l = s.slo_l; in.cap = s.cap;
    in.slo_a = s.slo_a;
    in.slo_raw = s.slo_a * hp.graph.amax;
    for (auto& h : in.held) h = jsv::NOT_HELD;
    return in;
}

// Tasks whose variant changes a downstream demand: an outgoing edge with unequal factors.
std::vector<uint32_t> influencers(const HostProblem& hp)
{
    std::vector<uint32_t> out;
    for (uint32_t t = 0; t < hp.T; ++t) {
        bool varies = false;
        for (uint32_t e = 0; e < hp.E; ++e)
            if (hp.src[e] == t)
                for (uint32_t v = 1; v < hp.V; ++v)
                    varies |= hp.fac[(size_t)e * hp.V + v] != hp.fac[(size_t)e * hp.V];
        if (varies) out.push_back(t);
    }
    return out;
}

constexpr uint64_t MAX_HELD_INSTANCES = 65536;

// Combinations of held variants per level; 0 if there are too many for one search.
uint64_t held_combinations(const HostProblem& hp, uint32_t n_levels)
{
    uint64_t n = 1;
    for (size_t k = influencers(hp).size(); k > 0; --k) {
        n *= hp.V;
        if (n * n_levels > MAX_HELD_INSTANCES) return 0;
    }
    return n;
}

// Is result a (one combination of held variants) better than the level's best so far, b?
bool held_better(int objective, const jsv_result& a, const jsv_result& b)
{
    if (!b.feasible) return true;
    if (objective && a.objective != b.objective) return a.objective > b.objective;
    if (a.cost_units != b.cost_units) return a.cost_units < b.cost_units;
    return a.full_index < b.full_index;
}

int ready_single(jsv_ctx* ctx)
{
    if (ctx->batch_mode) return JSV_E_STATE;
    HostProblem& hp = ctx->single;
    if (!hp.have_profile || !hp.have_dag) return JSV_E_STATE;
    if (hp.mult.size() != hp.T) return JSV_E_STATE;
    if (!hp.staged) {
        const int rc = stage_graph(hp, SpaceFlags{ctx->space_a, ctx->space_s, ctx->space_t});
        if (rc) return rc;
        ctx->dirty = true;
    }
    int rc = ensure_device(ctx);
    if (rc) return rc;
    if (ctx->dirty) { rc = upload_problems(ctx, &hp, 1); if (rc) return rc; }
    return JSV_OK;
}

}  // namespace

extern "C" {

JSV_API int jsv_create(jsv_ctx** out, int device, void* hip_stream)
{
    if (!out) return JSV_E_NULL;
    if (device < 0) return JSV_E_BADARG;
    jsv_ctx* ctx = new (std::nothrow) jsv_ctx();
    if (!ctx) return JSV_E_DEVICE;
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    *out = ctx;
    return JSV_OK;
}

JSV_API void jsv_destroy(jsv_ctx* ctx)
{
    if (!ctx) return;
    if (ctx->device_ready) {
        (void)hipSetDevice(ctx->device);
        (void)hipStreamSynchronize(ctx->stream);
        drop_graph(ctx);
        for (auto& e : ctx->ev) if (e) (void)hipEventDestroy(e);
        if (ctx->d_problems) (void)hipFree(ctx->d_problems);
        if (ctx->ws_own) (void)hipFree(ctx->ws_own);
        if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    }
    delete ctx;
}

JSV_API int jsv_last_hip_error(const jsv_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

JSV_API const char* jsv_error_string(int code)
{
    switch (code) {
    case JSV_OK: return "ok";
    case JSV_E_NULL: return "null pointer";
    case JSV_E_BADARG: return "argument out of range";
    case JSV_E_CYCLE: return "task graph has a cycle";
    case JSV_E_OVERFLOW: return "latency, cost or search space does not fit";
    case JSV_E_STATE: return "profile/graph missing or inconsistent";
    case JSV_E_WORKSPACE: return "workspace too small";
    case JSV_E_DEVICE: return "HIP call failed";
    case JSV_E_INTERNAL: return "enumeration and rescoring disagree";
    default: return "unknown error";
    }
}

JSV_API int jsv_set_objective(jsv_ctx* ctx, int mode, double alpha, double beta)
{
    if (!ctx) return JSV_E_NULL;
    if (mode != 0 && mode != 1) return JSV_E_BADARG;
    if (!(alpha >= 0.0) || !(beta >= 0.0) || std::isinf(alpha) || std::isinf(beta)) return JSV_E_BADARG;
    ctx->objective = mode; ctx->alpha = alpha; ctx->beta = beta;
    return JSV_OK;
}

JSV_API int jsv_set_search_space(jsv_ctx* ctx, int accuracy_scaling, int spatial_partitioning, int graph_informed)
{
    if (!ctx) return JSV_E_NULL;
    ctx->space_a = accuracy_scaling != 0;
    ctx->space_s = spatial_partitioning != 0;
    ctx->space_t = graph_informed != 0;
    // staged graphs carry the restrictions: stage and upload again before the next search
    ctx->single.staged = false;
    for (auto& hp : ctx->batch) {
        const int rc = stage_graph(hp, SpaceFlags{ctx->space_a, ctx->space_s, ctx->space_t});
        if (rc) return rc;
    }
    ctx->dirty = true;
    return JSV_OK;
}

JSV_API int jsv_set_graph_mode(jsv_ctx* ctx, int on)
{
    if (!ctx) return JSV_E_NULL;
    if (on && ctx->stream == nullptr) return JSV_E_STATE;     // the default stream cannot be captured
    ctx->graph_mode = on != 0;
    if (!ctx->graph_mode && ctx->device_ready) { (void)hipSetDevice(ctx->device); drop_graph(ctx); }
    return JSV_OK;
}

JSV_API size_t jsv_workspace_bytes(const jsv_ctx* ctx, uint32_t n_levels, uint32_t prune_cap)
{
    if (!ctx || n_levels == 0) return 0;
    uint32_t t_max = 0, k_max = 0, c_max = 0;
    if (ctx->batch_mode) {
        for (size_t k = 0; k < ctx->batch.size(); ++k) {
            t_max = std::max(t_max, ctx->batch[k].T);
            c_max = std::max(c_max, ctx->batch[k].C);
            k_max = std::max(k_max, k_max_of(ctx->batch[k], ctx->batch_search[k].cap));
        }
        n_levels = (uint32_t)ctx->batch.size();
    } else {
        if (!ctx->single.have_profile) return 0;
        t_max = ctx->single.T; c_max = ctx->single.C; k_max = k_max_of(ctx->single, prune_cap);
        if (!ctx->single.fac.empty()) {
            const uint64_t n_sub = held_combinations(ctx->single, n_levels);
            if (n_sub == 0) return 0;
            n_levels = (uint32_t)(n_levels * n_sub);
        }
    }
    const uint32_t grid = ctx->grid ? ctx->grid : 256u * 8u;
    uint64_t mix_cells = 0;
    if (ctx->mix && !ctx->batch_mode) {
        mix_cells = (uint64_t)(ctx->single.capacity + 1) * c_max;
        k_max = prune_cap;
        if (prune_cap < 2 || mix_cells * t_max * n_levels > ((uint64_t)1 << 32)) return 0;
    }
    return make_layout(n_levels, t_max, k_max, c_max, grid, 0, mix_cells).total;
}

JSV_API int jsv_set_workspace(jsv_ctx* ctx, void* device_ptr, size_t bytes)
{
    if (!ctx) return JSV_E_NULL;
    if (device_ptr && ((uintptr_t)device_ptr % ALIGN) != 0) return JSV_E_BADARG;
    ctx->ws_lent = device_ptr;
    ctx->ws_lent_bytes = device_ptr ? bytes : 0;
    return JSV_OK;
}

JSV_API int jsv_load_profile(jsv_ctx* ctx, uint32_t T, uint32_t V, uint32_t P, uint32_t B,
                     const uint32_t* units, const uint32_t* batch,
                     const uint32_t* latency_us, const uint32_t* thr_mrps, const double* accuracy)
{
    if (!ctx) return JSV_E_NULL;
    HostProblem hp = ctx->batch_mode ? HostProblem() : ctx->single;
    const int rc = check_profile(T, V, P, B, units, batch, latency_us, thr_mrps, accuracy, hp);
    if (rc) return rc;
    if (hp.have_dag && hp.mult.size() != T) { hp.have_dag = false; }   // a graph of another size is dropped
    ctx->single = std::move(hp);
    ctx->batch_mode = false;
    ctx->batch.clear(); ctx->batch_search.clear();
    ctx->dirty = true;
    return JSV_OK;
}

JSV_API int jsv_set_dag(jsv_ctx* ctx, uint32_t T, uint32_t E, const uint16_t* src, const uint16_t* dst,
                const uint32_t* demand_mult_milli, uint32_t capacity_units, uint32_t queue_factor)
{
    if (!ctx) return JSV_E_NULL;
    if (ctx->batch_mode) { ctx->single = HostProblem(); ctx->batch_mode = false; ctx->batch.clear(); ctx->batch_search.clear(); }
    HostProblem& hp = ctx->single;
    if (hp.have_profile && hp.T != T) return JSV_E_STATE;
    HostProblem tmp = hp;
    const int rc = check_dag(T, E, src, dst, demand_mult_milli, capacity_units, queue_factor, tmp);
    if (rc) return rc;
    if (tmp.have_profile) {                       // stage now so that range errors surface here
        const int rs = stage_graph(tmp, SpaceFlags{ctx->space_a, ctx->space_s, ctx->space_t});
        if (rs) return rs;
    }
    hp = std::move(tmp);
    ctx->dirty = true;
    return JSV_OK;
}

JSV_API int jsv_search(jsv_ctx* ctx, const uint32_t* demand_mrps, uint32_t n_levels,
               uint32_t slo_latency_us, double slo_accuracy, uint32_t prune_cap,
               jsv_result* out, jsv_summary* summary)
{
    if (!ctx || !demand_mrps || !out) return JSV_E_NULL;
    if (n_levels == 0) return JSV_E_BADARG;
    if (ctx->batch_mode || !ctx->single.have_profile || !ctx->single.have_dag) return JSV_E_STATE;
    for (uint32_t l = 0; l < n_levels; ++l) {
        // (mixture mode has its own bounds on prune_cap, below)
        const int rc = check_search_args(ctx->single, demand_mrps[l], slo_accuracy, ctx->mix ? 0 : prune_cap);
        if (rc) return rc;
    }
    int rc = ready_single(ctx);
    if (rc) return rc;
    const HostProblem& hp = ctx->single;
    if (ctx->mix) {
        // Mixtures of two tuples: the options of a task live in a grid of (cost 0..S_avail) x
        // (latency classes <= C) cells per (level, task)
        if (!hp.fac.empty() || !ctx->space_t) return JSV_E_STATE;
        if (prune_cap < 2 || prune_cap > JSV_MAX_CHOICES || hp.capacity == 0 || hp.capacity > 65535) return JSV_E_BADARG;
        const uint64_t cells = (uint64_t)(hp.capacity + 1) * hp.C;
        if (cells * hp.T * n_levels > ((uint64_t)1 << 32)) return JSV_E_WORKSPACE;      // 28 B per cell
        std::vector<Instance> inst(n_levels);
        for (uint32_t l = 0; l < n_levels; ++l)
            inst[l] = make_instance(ctx, hp, 0, Search{demand_mrps[l], slo_latency_us, prune_cap, slo_accuracy});
        return run_search(ctx, inst, hp.T, prune_cap, hp.C, out, summary, cells);
    }
    if (!hp.fac.empty()) {
        // Per-variant factors: one instance per (level, combination of held variants), lowest
        // held task id = fastest digit; the level's result is the best over its combinations.
        if (!ctx->space_t) return JSV_E_STATE;
        const std::vector<uint32_t> inf = influencers(hp);
        const uint64_t n_sub = held_combinations(hp, n_levels);
        if (n_sub == 0) return JSV_E_BADARG;
        std::vector<Instance> inst((size_t)n_levels * n_sub);
        for (uint32_t l = 0; l < n_levels; ++l)
            for (uint64_t u = 0; u < n_sub; ++u) {
                Instance in = make_instance(ctx, hp, 0, Search{demand_mrps[l], slo_latency_us, prune_cap, slo_accuracy});
                uint64_t rest = u;
                for (uint32_t t : inf) { in.held[t] = (uint16_t)(rest % hp.V); rest /= hp.V; }
                inst[(size_t)l * n_sub + u] = in;
            }
        std::vector<jsv_result> sub(inst.size());
        rc = run_search(ctx, inst, hp.T, k_max_of(hp, prune_cap), hp.C, sub.data(), summary);
        if (rc) return rc;
        int32_t best_level = -1;
        uint32_t max_demand = 0;
        for (uint32_t l = 0; l < n_levels; ++l) {
            jsv_result best;
            std::memset(&best, 0, sizeof best);
            best.index = best.full_index = ~0ull;
            best.cost_units = 0x7FFFFFFF;
            uint64_t evaluated = 0;
            uint32_t flags = 0;
            for (uint64_t u = 0; u < n_sub; ++u) {
                const jsv_result& r = sub[(size_t)l * n_sub + u];
                evaluated += r.evaluated;
                flags |= r.flags;
                if (!r.feasible) continue;
                if (r.full_index == ~0ull) return JSV_E_OVERFLOW;
                if (held_better(ctx->objective, r, best)) best = r;
            }
            best.index = best.full_index;
            best.evaluated = evaluated;
            best.flags = flags;
            out[l] = best;
            if (best.feasible && (best_level < 0 || demand_mrps[l] > max_demand)) { best_level = (int32_t)l; max_demand = demand_mrps[l]; }
        }
        if (summary) { summary->best_level = best_level; summary->max_demand_mrps = max_demand; }
        return JSV_OK;
    }
    std::vector<Instance> inst(n_levels);
    for (uint32_t l = 0; l < n_levels; ++l)
        inst[l] = make_instance(ctx, hp, 0, Search{demand_mrps[l], slo_latency_us, prune_cap, slo_accuracy});
    return run_search(ctx, inst, hp.T, k_max_of(hp, prune_cap), hp.C, out, summary);
}

JSV_API int jsv_search_static(jsv_ctx* ctx, const uint32_t* demand_mrps, uint32_t n_levels,
                      uint32_t slo_latency_us, double slo_accuracy, uint32_t prune_cap,
                      jsv_result* out, jsv_summary* summary)
{
    if (!ctx || !demand_mrps || !out) return JSV_E_NULL;
    if (n_levels == 0) return JSV_E_BADARG;
    HostProblem& hp = ctx->single;
    if (ctx->batch_mode || !hp.have_profile || !hp.have_dag || hp.mult.size() != hp.T) return JSV_E_STATE;
    if (ctx->mix || !hp.fac.empty() || ctx->graph_mode) return JSV_E_STATE;
    for (uint32_t l = 0; l < n_levels; ++l) {
        const int rc = check_search_args(hp, demand_mrps[l], slo_accuracy, prune_cap);
        if (rc) return rc;
    }
    if (!hp.staged) {
        const int rc = stage_graph(hp, SpaceFlags{ctx->space_a, ctx->space_s, ctx->space_t});
        if (rc) return rc;
        ctx->dirty = true;                      // for the allocating entry points: their blob is stale too
    }
    // does it fit the static array?  (checked before any device call; per-block partial results
    // are sized for the device's compute units, 256 before the first device call)
    const uint32_t k_max = k_max_of(hp, prune_cap);
    const size_t blob_bytes = build_blob(&hp, 1, nullptr, nullptr);
    const uint32_t grid = ctx->grid ? ctx->grid : 256u * 8u;
    if (blob_bytes + make_layout(n_levels, hp.T, k_max, hp.C, grid, 0, 0).total > JSV_STATIC_SCRATCH_BYTES)
        return JSV_E_WORKSPACE;
    int rc = ensure_device(ctx);
    if (rc) return rc;
    StaticArena sa{nullptr, blob_bytes};
    rc = static_scratch(ctx, &sa.base);
    if (rc) return rc;
    // the array is shared by every context on this GPU: the blob goes up with every call
    std::vector<unsigned char> blob;
    build_blob(&hp, 1, sa.base, &blob);
    HIP_TRY(ctx, hipMemcpyAsync(sa.base, blob.data(), blob_bytes, hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));      // blob is a local buffer
    std::vector<Instance> inst(n_levels);
    for (uint32_t l = 0; l < n_levels; ++l)
        inst[l] = make_instance(ctx, hp, 0, Search{demand_mrps[l], slo_latency_us, prune_cap, slo_accuracy});
    return run_search(ctx, inst, hp.T, k_max, hp.C, out, summary, 0, &sa);
}

JSV_API int jsv_set_bounds(jsv_ctx* ctx, int on)
{
    if (!ctx) return JSV_E_NULL;
    ctx->bounds = on != 0;
    return JSV_OK;
}

JSV_API int jsv_set_geometry(jsv_ctx* ctx, int blocks_per_cu, int lanes_percent)
{
    if (!ctx) return JSV_E_NULL;
    if (blocks_per_cu < 0 || blocks_per_cu > 8 || lanes_percent < 0 || lanes_percent > 1600) return JSV_E_BADARG;
    ctx->geo_blocks = blocks_per_cu;
    ctx->geo_lanes_percent = lanes_percent;
    return JSV_OK;
}

JSV_API int jsv_set_mixtures(jsv_ctx* ctx, int on)
{
    if (!ctx) return JSV_E_NULL;
    ctx->mix = on != 0;
    return JSV_OK;
}

JSV_API int jsv_set_factors(jsv_ctx* ctx, const uint32_t* factor_milli)
{
    if (!ctx) return JSV_E_NULL;
    HostProblem& hp = ctx->single;
    if (ctx->batch_mode || !hp.have_profile || !hp.have_dag) return JSV_E_STATE;
    if (!factor_milli) {
        if (!hp.fac.empty()) { hp.fac.clear(); ctx->dirty = true; }
        return JSV_OK;
    }
    if (hp.E == 0) return JSV_E_BADARG;
    const size_t n = (size_t)hp.E * hp.V;
    for (size_t k = 0; k < n; ++k)
        if (factor_milli[k] == 0 || factor_milli[k] > JSV_MAX_FACTOR_MILLI) return JSV_E_BADARG;
    // the winner's index is reported in the full space: C^T must fit 64 bits
    unsigned __int128 full = 1;
    for (uint32_t t = 0; t < hp.T; ++t) { full *= hp.C; if (full >> 64) return JSV_E_OVERFLOW; }
    hp.fac.assign(factor_milli, factor_milli + n);
    ctx->dirty = true;
    return JSV_OK;
}

JSV_API int jsv_eval_candidates(jsv_ctx* ctx, uint32_t demand_mrps, uint32_t slo_latency_us,
                        double slo_accuracy, uint32_t prune_cap,
                        const uint64_t* index, uint32_t n,
                        uint32_t* latency_us, uint32_t* replicas, int32_t* cost,
                        double* accuracy, uint8_t* mask)
{
    if (!ctx || !index || !latency_us || !replicas || !cost || !accuracy || !mask) return JSV_E_NULL;
    if (ctx->batch_mode || !ctx->single.have_profile || !ctx->single.have_dag) return JSV_E_STATE;
    if (!ctx->single.fac.empty() || ctx->mix) return JSV_E_STATE;   // no single list of choice ids there
    int rc = check_search_args(ctx->single, demand_mrps, slo_accuracy, prune_cap);
    if (rc) return rc;
    if (n == 0) return JSV_OK;
    rc = ready_single(ctx);
    if (rc) return rc;
    const HostProblem& hp = ctx->single;
    const uint32_t T = hp.T, k_max = k_max_of(hp, prune_cap);
    if (jsv::prune_lds_bytes(hp.C) > 64 * 1024) return JSV_E_BADARG;
    const Layout L = make_layout(1, T, k_max, hp.C, ctx->grid, n);
    unsigned char* ws = nullptr;
    rc = get_workspace(ctx, L.total, &ws);
    if (rc) return rc;
    Instance in = make_instance(ctx, hp, 0, Search{demand_mrps, slo_latency_us, prune_cap, slo_accuracy});

    jsv::Plan pl = make_plan(ctx, ctx->d_problems, L, ws, 1, T, k_max, hp.C, 0);
    pl.grid = ctx->grid; pl.lanes_wanted = 64;

    unsigned char* e = ws + L.eval;
    uint64_t* d_index = (uint64_t*)e;          e += align_up(sizeof(uint64_t) * n);
    double* d_acc = (double*)e;                e += align_up(sizeof(double) * n);
    uint32_t* d_lat = (uint32_t*)e;            e += align_up(sizeof(uint32_t) * n);
    int32_t* d_cost = (int32_t*)e;             e += align_up(sizeof(int32_t) * n);
    uint32_t* d_rep = (uint32_t*)e;            e += align_up(sizeof(uint32_t) * (size_t)n * T);
    uint8_t* d_mask = (uint8_t*)e;             e += align_up(n);
    uint32_t* d_bad = (uint32_t*)e;

    hipStream_t st = ctx->stream;
    uint32_t bad = 0;
    HIP_TRY(ctx, hipMemcpyAsync(pl.inst, &in, sizeof in, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(d_index, index, sizeof(uint64_t) * n, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipMemcpyAsync(d_bad, &bad, sizeof bad, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));      // sources are caller / stack memory
    HIP_TRY(ctx, jsv::launch_prune_plan_scan(pl, st));
    HIP_TRY(ctx, jsv::launch_eval(pl, d_index, n, d_lat, d_rep, d_cost, d_acc, d_mask, d_bad, st));
    Instance back;
    HIP_TRY(ctx, hipMemcpyAsync(&back, pl.inst, sizeof back, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(&bad, d_bad, sizeof bad, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(latency_us, d_lat, sizeof(uint32_t) * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(replicas, d_rep, sizeof(uint32_t) * (size_t)n * T, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(cost, d_cost, sizeof(int32_t) * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(accuracy, d_acc, sizeof(double) * n, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(mask, d_mask, n, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    if (back.flags & jsv::F_OVERFLOW) return JSV_E_OVERFLOW;
    if (bad) return JSV_E_BADARG;
    return JSV_OK;
}

JSV_API int jsv_get_pruned(jsv_ctx* ctx, uint32_t demand_mrps, uint32_t slo_latency_us,
                   uint32_t prune_cap, uint32_t task,
                   uint16_t* choice_ids, uint32_t* K, uint32_t* truncated)
{
    if (!ctx || !choice_ids || !K || !truncated) return JSV_E_NULL;
    if (ctx->batch_mode || !ctx->single.have_profile || !ctx->single.have_dag) return JSV_E_STATE;
    if (!ctx->single.fac.empty() || ctx->mix) return JSV_E_STATE;   // no single list of choice ids there
    if (task >= ctx->single.T) return JSV_E_BADARG;
    int rc = check_search_args(ctx->single, demand_mrps, 0.0, prune_cap);
    if (rc) return rc;
    rc = ready_single(ctx);
    if (rc) return rc;
    const HostProblem& hp = ctx->single;
    const uint32_t T = hp.T, k_max = k_max_of(hp, prune_cap);
    if (jsv::prune_lds_bytes(hp.C) > 64 * 1024) return JSV_E_BADARG;
    const Layout L = make_layout(1, T, k_max, hp.C, ctx->grid, 0);
    unsigned char* ws = nullptr;
    rc = get_workspace(ctx, L.total, &ws);
    if (rc) return rc;
    Instance in = make_instance(ctx, hp, 0, Search{demand_mrps, slo_latency_us, prune_cap, 0.0});
    jsv::Plan pl = make_plan(ctx, ctx->d_problems, L, ws, 1, T, k_max, hp.C, 0);
    pl.grid = ctx->grid; pl.lanes_wanted = 64;
    hipStream_t st = ctx->stream;
    HIP_TRY(ctx, hipMemcpyAsync(pl.inst, &in, sizeof in, hipMemcpyHostToDevice, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    HIP_TRY(ctx, jsv::launch_prune_plan_scan(pl, st));
    Instance back;
    std::vector<jsv::Entry> ent(k_max);
    HIP_TRY(ctx, hipMemcpyAsync(&back, pl.inst, sizeof back, hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipMemcpyAsync(ent.data(), pl.entries + (size_t)task * k_max, sizeof(jsv::Entry) * k_max,
                                hipMemcpyDeviceToHost, st));
    HIP_TRY(ctx, hipStreamSynchronize(st));
    const uint32_t k = back.K[task];
    for (uint32_t d = 0; d < k; ++d) choice_ids[d] = (uint16_t)ent[d].choice;
    *K = k;
    *truncated = (back.trunc_mask >> task) & 1u;
    return JSV_OK;
}

JSV_API int jsv_load_batch(jsv_ctx* ctx, const jsv_problem* problems, uint32_t n, uint32_t* bad)
{
    if (!ctx || !problems) return JSV_E_NULL;
    if (n == 0) return JSV_E_BADARG;
    std::vector<HostProblem> hps(n);
    std::vector<Search> ss(n);
    for (uint32_t k = 0; k < n; ++k) {
        const jsv_problem& p = problems[k];
        if (bad) *bad = k;
        int rc = check_profile(p.T, p.V, p.P, p.B, p.units, p.batch, p.latency_us, p.thr_mrps, p.accuracy, hps[k]);
        if (rc) return rc;
        rc = check_dag(p.T, p.E, p.src, p.dst, p.demand_mult_milli, p.capacity_units, p.queue_factor, hps[k]);
        if (rc) return rc;
        rc = stage_graph(hps[k], SpaceFlags{ctx->space_a, ctx->space_s, ctx->space_t});
        if (rc) return rc;
        rc = check_search_args(hps[k], p.demand_mrps, p.slo_accuracy, p.prune_cap);
        if (rc) return rc;
        ss[k] = Search{p.demand_mrps, p.slo_latency_us, p.prune_cap, p.slo_accuracy};
    }
    if (bad) *bad = 0;
    ctx->batch.swap(hps);
    ctx->batch_search.swap(ss);
    ctx->batch_mode = true;
    ctx->single = HostProblem();
    ctx->dirty = true;
    int rc = ensure_device(ctx);
    if (rc) return rc;
    return upload_problems(ctx, ctx->batch.data(), n);
}

JSV_API int jsv_search_loaded_batch(jsv_ctx* ctx, jsv_result* out, jsv_summary* summary)
{
    if (!ctx || !out) return JSV_E_NULL;
    if (!ctx->batch_mode || ctx->batch.empty() || ctx->mix) return JSV_E_STATE;
    int rc = ensure_device(ctx);
    if (rc) return rc;
    if (ctx->dirty) { rc = upload_problems(ctx, ctx->batch.data(), (uint32_t)ctx->batch.size()); if (rc) return rc; }
    const uint32_t n = (uint32_t)ctx->batch.size();
    std::vector<Instance> inst(n);
    uint32_t t_max = 0, k_max = 0, c_max = 0;
    for (uint32_t k = 0; k < n; ++k) {
        inst[k] = make_instance(ctx, ctx->batch[k], k, ctx->batch_search[k]);
        t_max = std::max(t_max, ctx->batch[k].T);
        c_max = std::max(c_max, ctx->batch[k].C);
        k_max = std::max(k_max, k_max_of(ctx->batch[k], ctx->batch_search[k].cap));
    }
    return run_search(ctx, inst, t_max, k_max, c_max, out, summary);
}

JSV_API int jsv_search_batch(jsv_ctx* ctx, const jsv_problem* problems, uint32_t n, jsv_result* out)
{
    const int rc = jsv_load_batch(ctx, problems, n, nullptr);
    if (rc) return rc;
    return jsv_search_loaded_batch(ctx, out, nullptr);
}

}  // extern "C"
