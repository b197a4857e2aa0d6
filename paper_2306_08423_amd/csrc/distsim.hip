// C ABI of the batched DistSim strategy evaluator (see include/distsim.h).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "distsim.h"
#include "kernels_build.hpp"
#include "kernels_ingest.hpp"
#include "kernels_search.hpp"
#include "kernels_explicit.hpp"
#include "kernels_schedule.hpp"
#include "kernels_simulate.hpp"
#include "kernels_timeline.hpp"
#include "kernels_virtual.hpp"

using namespace distsim;

// Scratch of distsim_search_static: the per-workgroup partial results of the argmin, in a device
// array of the library itself, so that this entry point needs no memory from anybody.  In host code
// the name is only a handle: the array's device address comes from hipGetSymbolAddress, once per
// context (with the context's device current), and only that pointer is handed to kernels.
static __device__ __align__(256) unsigned char scratch[kSearchMaxBlocks * sizeof(Best)];

struct TimedLaunch {
    hipEvent_t start, stop;
};

struct distsim_ctx {
    int device = 0;
    int num_cus = 256;
    int64_t split_min_items = kSplitMinItems;   // lists of fewer wave-items go through k_simulate alone
    int64_t grid_per_cu = 128;                  // groups of four wavefronts per CU of the sweep launches (at most)
    // k_simulate_gpipe runs next to k_simulate on a stream of the context (default priority),
    // forked from and joined to the caller's stream with the two events
    hipStream_t side = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    void* static_scratch = nullptr;          // device address of `scratch` on this context's device
    std::string static_scratch_err;          // why it could not be taken (empty = taken)
    std::string err;
    bool timing = false;
    std::vector<TimedLaunch> rec[DISTSIM_K_COUNT];
    std::vector<TimedLaunch> pool;      // recycled event pairs
};

static const char* kKernelNames[DISTSIM_K_COUNT] = {
    "k_layer_tables", "k_decode", "k_bins", "k_scatter",
    "k_stage_events", "k_sim_init", "k_simulate", "k_search", "k_timeline",
    "k_dedup", "k_comm_event_times", "k_bubbles", "k_simulate_virtual",
    "k_timeline_virtual", "k_simulate_gpipe", "k_simulate_explicit", "k_timeline_explicit",
    "k_compile_schedules", "k_timeline_gpipe",
};

static int fail(distsim_ctx* ctx, int code, const std::string& msg) {
    if (ctx) ctx->err = msg;
    return code;
}

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail(ctx, DISTSIM_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    } while (0)

namespace {

// Brackets a group of launches with HIP events on the caller's stream when timing is on.
struct Timer {
    distsim_ctx* ctx;
    hipStream_t stream;
    int kid;
    TimedLaunch tl{};
    bool on = false;
    Timer(distsim_ctx* c, hipStream_t s, int k) : ctx(c), stream(s), kid(k) {
        if (!ctx->timing) return;
        if (!ctx->pool.empty()) { tl = ctx->pool.back(); ctx->pool.pop_back(); }
        else if (hipEventCreate(&tl.start) != hipSuccess || hipEventCreate(&tl.stop) != hipSuccess) return;
        on = hipEventRecord(tl.start, stream) == hipSuccess;
    }
    ~Timer() {
        if (!on) return;
        (void)hipEventRecord(tl.stop, stream);
        ctx->rec[kid].push_back(tl);
    }
};

ClusterDev to_dev(const distsim_cluster& c);
ClusterDev cl_dev(const distsim_cluster& c) { return to_dev(c); }
ClusterDev to_dev(const distsim_cluster& c) {
    ClusterDev d;
    d.num_devices = c.num_devices;
    d.gpus_per_node = c.gpus_per_node;
    d.alpha[0] = c.alpha_ns[0]; d.alpha[1] = c.alpha_ns[1];
    d.beta[0] = c.beta_bytes_per_ns[0]; d.beta[1] = c.beta_bytes_per_ns[1];
    d.bucket = c.dp_bucket_bytes;
    d.blocking = c.p2p_blocking;
    d.inv_gpus_per_node = 1.0 / (double)c.gpus_per_node;
    d.gpus_per_node_f = (double)c.gpus_per_node;
    d.inv_bucket = c.dp_bucket_bytes > 0 ? 1.0 / (double)c.dp_bucket_bytes : 0.0;
    return d;
}

bool cluster_ok(const distsim_cluster* c) {
    return c && c->num_devices >= 1 && c->gpus_per_node >= 1 && c->alpha_ns[0] >= 0 && c->alpha_ns[1] >= 0 &&
           c->beta_bytes_per_ns[0] >= 1 && c->beta_bytes_per_ns[1] >= 1 && c->dp_bucket_bytes >= 0 &&
           c->p2p_blocking >= 0 && c->p2p_blocking <= 2;
}

// Bounds that keep every product of the collective formulas within 63 bits (with table entries
// below 2^40) and every bucket count exact in fp64.
bool cluster_in_range(const distsim_cluster* c) {
    const int64_t a = (int64_t)1 << 40, b = (int64_t)1 << 32;
    return c->num_devices <= (1 << 22) && c->alpha_ns[0] < a && c->alpha_ns[1] < a && c->beta_bytes_per_ns[0] < b &&
           c->beta_bytes_per_ns[1] < b && c->dp_bucket_bytes < ((int64_t)1 << 53);
}

// Makes the context's device current for the duration of a call and restores the caller's.
struct DeviceScope {
    int prev = -1;
    hipError_t err;
    explicit DeviceScope(int device) {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        err = prev == device ? hipSuccess : hipSetDevice(device);
        if (prev == device) prev = -1;                           // nothing to restore
    }
    ~DeviceScope() { if (prev >= 0) (void)hipSetDevice(prev); }
};

CandDev cand_dev(const distsim_candidates* cand) {
    return CandDev{cand->dp, cand->tp, cand->pp, cand->m, cand->schedule, cand->part_off, cand->part_pool,
                   cand->part_pool ? cand->part_pool_len : 0, cand->chunks,
                   cand->schedule_off && cand->schedule_words ? cand->n_schedules : 0, cand->schedule_off,
                   cand->schedule_words, cand->schedule_words_len};
}

bool cand_arrays_ok(const distsim_candidates* cand) {
    return cand->dp && cand->tp && cand->pp && cand->m && cand->schedule && cand->part_off;
}

// What the calls after event generation know of the cost table: its shape and, through the copy in
// the workspace, the tensor-parallel size of every variant.
CostsDev costs_after_build(const distsim_events* ev, const Workspace& ws) {
    return CostsDev{ev->L, ev->V, ws.vtp, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
}

// Layout of the single allocation of distsim_events_bind; base may be null (size query).
size_t carve_events(distsim_events* ev, void* base, int32_t L, int32_t V, int64_t C, int64_t stage_cap, bool table) {
    size_t off = 0;
    char* b = (char*)base;
    auto take = [&](size_t bytes) { void* p = b ? (void*)(b + off) : nullptr; off += align256(bytes); return p; };
    const size_t Cc = (size_t)(C > 0 ? C : 1), cap = (size_t)(stage_cap > 0 ? stage_cap : 1);
    Workspace w;
    const size_t wbytes = carve(w, nullptr, L, V, C);
    void* status = take(Cc * 4);
    void* pos = take(Cc * 8);
    void* nev = take(Cc * 8);
    void* wsp = take(wbytes);
    void* tab = table ? take(cap * DISTSIM_NCOLS * 8) : nullptr;
    void* lay = table ? take(cap * 4) : nullptr;
    if (ev) {
        ev->stage_cap = stage_cap; ev->L = L; ev->V = V;
        ev->status = (int32_t*)status; ev->stage_pos = (int64_t*)pos; ev->num_events = (int64_t*)nev;
        ev->stage_tab = (int64_t*)tab; ev->stage_layers = (int32_t*)lay;
        ev->workspace = wsp; ev->workspace_bytes = wbytes; ev->num_candidates = 0;
    }
    return off;
}

// Waves that sweep the wave-items: enough to fill every SIMD, never more than one per candidate.
// Grid of k_simulate: a wavefront takes two items per turn and items differ a lot in length, so
// the grid is many times what is resident at once and the dispatcher evens the load out.
int simulate_grid(const distsim_ctx* ctx, int64_t C) {
    const int64_t want = (int64_t)ctx->num_cus * ctx->grid_per_cu;
    const int64_t need = (C + 7) / 8;                         // in groups of 4 wavefronts (the launch multiplies by 256 / kSimBlock), 2 items per wavefront
    return (int)(need < want ? (need < 1 ? 1 : need) : want);
}

// k_simulate: the whole grid for a list that it simulates alone, less for a list long enough to
// be shared with k_simulate_gpipe (wavefronts stride over their kernel's pairs, so any split of
// the items is covered by any grid)
int general_grid(const distsim_ctx* ctx, int64_t C) {
    const int g = simulate_grid(ctx, C);
    return C >= ctx->split_min_items && g >= 2 ? g / 2 : g;
}

// k_simulate_gpipe takes at most the GPipe half of the items (a wavefront strides over its
// kernel's pairs, so any split of the items is covered)
int gpipe_grid(const distsim_ctx* ctx, int64_t C) {
    const int g = simulate_grid(ctx, C) / 2;
    return g < 1 ? 1 : g;
}

int item_grid(const distsim_ctx* ctx, int64_t C) {
    const int64_t want = (int64_t)ctx->num_cus * 8;           // blocks of 4 waves: 8 waves per SIMD
    const int64_t need = (C + 3) / 4;
    return (int)(need < want ? (need < 1 ? 1 : need) : want);
}

}  // namespace

extern "C" {

int distsim_create(distsim_ctx** out, int hip_device) {
    if (!out) return DISTSIM_EINVAL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || hip_device < 0 || hip_device >= n) return DISTSIM_EHIP;
    distsim_ctx* ctx = new distsim_ctx();
    ctx->device = hip_device;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, hip_device) == hipSuccess && prop.multiProcessorCount > 0)
        ctx->num_cus = prop.multiProcessorCount;
    int prev = 0;
    const bool had = hipGetDevice(&prev) == hipSuccess;
    const bool made = hipSetDevice(hip_device) == hipSuccess &&
                      hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) == hipSuccess &&
                      hipEventCreateWithFlags(&ctx->fork, hipEventDisableTiming) == hipSuccess &&
                      hipEventCreateWithFlags(&ctx->join, hipEventDisableTiming) == hipSuccess;
    if (made) {
        // every device holds its own copy of the array at its own address
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e == hipSuccess && p) ctx->static_scratch = p;
        else ctx->static_scratch_err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
    }
    if (had) (void)hipSetDevice(prev);
    if (!made) { distsim_destroy(ctx); return DISTSIM_EHIP; }
    if (const char* e = getenv("DISTSIM_SPLIT_MIN_ITEMS")) {
        char* end = nullptr;
        const long long v = strtoll(e, &end, 10);
        if (end != e && v >= 0) ctx->split_min_items = v;
    }
    *out = ctx;
    return DISTSIM_OK;
}

void distsim_destroy(distsim_ctx* ctx) {
    if (!ctx) return;
    for (auto& v : ctx->rec) for (auto& t : v) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
    for (auto& t : ctx->pool) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
    if (ctx->fork) (void)hipEventDestroy(ctx->fork);
    if (ctx->join) (void)hipEventDestroy(ctx->join);
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    delete ctx;
}

const char* distsim_last_error(const distsim_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int64_t distsim_stage_entries(int64_t C) { return C < 0 ? 0 : C * kWave + (kClasses * kWave); }

size_t distsim_workspace_bytes(int32_t L, int32_t V, int64_t C) {
    if (L < 1 || L > DISTSIM_MAX_L || V < 1 || V > DISTSIM_MAX_V || C < 0 || C > 0x7fffffff) return 0;
    Workspace w;
    return carve(w, nullptr, L, V, C);
}

size_t distsim_events_bytes(const distsim_costs* costs, int64_t C, int64_t stage_cap, int with_stage_table) {
    if (!costs || stage_cap < 0 || distsim_workspace_bytes(costs->L, costs->V, C) == 0) return 0;
    return carve_events(nullptr, nullptr, costs->L, costs->V, C, stage_cap, with_stage_table != 0);
}

int distsim_events_bind(distsim_events* ev, void* memory, size_t memory_bytes, const distsim_costs* costs, int64_t C,
                        int64_t stage_cap, int with_stage_table) {
    if (!ev || !memory || !costs || stage_cap < 0 || C < 0 || ((uintptr_t)memory & 255) != 0) return DISTSIM_EINVAL;
    const size_t need = distsim_events_bytes(costs, C, stage_cap, with_stage_table);
    if (need == 0) return DISTSIM_ELIMIT;
    if (memory_bytes < need) return DISTSIM_EINVAL;
    (void)carve_events(ev, memory, costs->L, costs->V, C, stage_cap, with_stage_table != 0);
    return DISTSIM_OK;
}

int distsim_build_events(distsim_ctx* ctx, const distsim_costs* costs, const distsim_cluster* cluster,
                         const distsim_candidates* cand, int64_t C, distsim_events* out, void* hip_stream) {
    if (!ctx) return DISTSIM_EINVAL;
    if (!costs || !cluster || !cand || !out) return fail(ctx, DISTSIM_EINVAL, "null argument");
    if (costs->L < 1 || costs->L > DISTSIM_MAX_L || costs->V < 1 || costs->V > DISTSIM_MAX_V)
        return fail(ctx, DISTSIM_ELIMIT, "cost table shape outside 1 <= L <= 255, 1 <= V <= 16");
    if (C < 0) return fail(ctx, DISTSIM_EINVAL, "negative candidate count");
    if (C > 0x7fffffff) return fail(ctx, DISTSIM_ELIMIT, "candidate count outside [0, 2^31)");
    if (!cluster_ok(cluster)) return fail(ctx, DISTSIM_EINVAL, "cluster description out of range");
    if (!cluster_in_range(cluster)) return fail(ctx, DISTSIM_ERANGE, "cluster: alpha >= 2^40, beta >= 2^32, bucket >= 2^53 or more than 2^22 devices");
    if (!costs->variant_tp || !costs->fwd_comp_ns || !costs->bwd_comp_ns || !costs->fwd_comm_ns ||
        !costs->bwd_comm_ns || !costs->act_bytes || !costs->grad_bytes)
        return fail(ctx, DISTSIM_EINVAL, "null cost column");
    if (!out->workspace || out->stage_cap < 0)
        return fail(ctx, DISTSIM_EINVAL, "events: null workspace or negative stage_cap");
    if (C > 0 && (!cand->dp || !cand->tp || !cand->pp || !cand->m || !cand->schedule || !cand->part_off ||
                  !out->status || !out->num_events || !out->stage_pos ||
                  ((out->stage_tab == nullptr) != (out->stage_layers == nullptr))))
        return fail(ctx, DISTSIM_EINVAL, "null candidate or events array");
    if (((uintptr_t)out->workspace & 255) != 0) return fail(ctx, DISTSIM_EINVAL, "workspace must be 256-byte aligned");
    Workspace ws;
    const size_t need = carve(ws, out->workspace, costs->L, costs->V, C);
    if (out->workspace_bytes < need) return fail(ctx, DISTSIM_EINVAL, "workspace too small");

    DeviceScope dev(ctx->device);
    HIP_TRY(dev.err);
    hipStream_t st = (hipStream_t)hip_stream;
    CostsDev co{costs->L, costs->V, costs->variant_tp, costs->fwd_comp_ns, costs->bwd_comp_ns, costs->fwd_comm_ns,
                costs->bwd_comm_ns, costs->act_bytes, costs->grad_bytes, costs->a2a_bytes};
    const ClusterDev cl = to_dev(*cluster);
    const CandDev ca = cand_dev(cand);
    EventsDev ev{out->stage_cap, out->status, out->stage_pos, out->stage_tab, out->stage_layers, out->num_events};
    out->L = costs->L;
    out->V = costs->V;
    out->num_candidates = C;

    // The layer tables do not depend on the candidates and nothing before k_stage_events reads
    // them: for a long list they are built on the context's stream next to decode / bins / scatter.
    const bool beside = C >= ctx->split_min_items;
    // The explicit schedules are turned into programs once, for all the candidates that use them
    // (after k_layer_tables on the same stream, which clears the count of schedules without one).
    auto compile_schedules = [&](hipStream_t s) {
        if (!cand->chunks || ca.n_schedules <= 0) return;
        Timer t(ctx, s, DISTSIM_K_COMPILE_SCHEDULES);
        const int64_t ids = ca.n_schedules < kSchedCap ? ca.n_schedules : kSchedCap;
        hipLaunchKernelGGL(k_compile_schedules, dim3((unsigned)ids), dim3(kWave), 0, s, ca, ws);
    };
    if (beside) {
        HIP_TRY(hipEventRecord(ctx->fork, st));
        HIP_TRY(hipStreamWaitEvent(ctx->side, ctx->fork, 0));
        {
            Timer t(ctx, ctx->side, DISTSIM_K_LAYER_TABLES);
            hipLaunchKernelGGL(k_layer_tables, dim3(costs->V * kMaxPP), dim3(kWave), 0, ctx->side, co, cl, ws);
        }
        compile_schedules(ctx->side);
        HIP_TRY(hipEventRecord(ctx->join, ctx->side));
        hipLaunchKernelGGL(k_clear_bins, dim3((kBins + 255) / 256), dim3(256), 0, st, ws);
    } else {
        Timer t(ctx, st, DISTSIM_K_LAYER_TABLES);
        hipLaunchKernelGGL(k_layer_tables, dim3(costs->V * kMaxPP), dim3(kWave), 0, st, co, cl, ws);
        hipLaunchKernelGGL(k_clear_bins, dim3((kBins + 255) / 256), dim3(256), 0, st, ws);
        compile_schedules(st);
    }
    if (C > 0) {
        Timer t(ctx, st, DISTSIM_K_DECODE);
        hipLaunchKernelGGL(k_decode, dim3((int)((C + kDecodeChunk - 1) / kDecodeChunk)), dim3(kDecodeBlock), 0, st,
                           co, cl, ca, C, ws, ev);
    }
    {
        Timer t(ctx, st, DISTSIM_K_BINS);
        hipLaunchKernelGGL(k_bins, dim3(1), dim3(kBinsBlock), 0, st, ws, out->stage_cap);
    }
    {
        // also for C == 0: the first threads fill the order tables of the sweep kernels (their totals)
        Timer t(ctx, st, DISTSIM_K_SCATTER);
        const int64_t threads = C > ws.order_cap ? C : ws.order_cap;
        // with a bucketed all-reduce: the classes whose stages hold 16 layers or more go first (their epilogues are long)
        int first_whole = kClasses;
        if (cluster->dp_bucket_bytes > 0)
            for (int k = kClasses - 1; k >= 0 && ((int64_t)costs->L << k) >= 16 * kWave; k--) first_whole = k;
        hipLaunchKernelGGL(k_scatter, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, ca, C, ws, ev,
                           C >= ctx->split_min_items ? 0 : INT64_MAX, first_whole);     // two launches: the same rule as distsim_simulate's, by candidates
    }
    if (beside) HIP_TRY(hipStreamWaitEvent(st, ctx->join, 0));       // what follows on the caller's stream sees the tables
    if (C > 0) {
        if (out->stage_tab && out->stage_cap > 0) {
            Timer t(ctx, st, DISTSIM_K_STAGE_EVENTS);
            hipLaunchKernelGGL(k_stage_events, dim3(item_grid(ctx, C)), dim3(256), 0, st, co, cl, ca, ws, ev);
        }
    }
    HIP_TRY(hipGetLastError());
    return DISTSIM_OK;
}

int distsim_simulate(distsim_ctx* ctx, const distsim_cluster* cluster, const distsim_candidates* cd,
                     const distsim_events* events, int64_t C, int64_t* batch_ns, int64_t* comp_busy_ns,
                     int64_t* comm_busy_ns, double* util, void* hip_stream) {
    if (!ctx) return DISTSIM_EINVAL;
    if (!cluster || !events || !cd) return fail(ctx, DISTSIM_EINVAL, "null argument");
    if (!cluster_ok(cluster)) return fail(ctx, DISTSIM_EINVAL, "cluster description out of range");
    if (!cluster_in_range(cluster)) return fail(ctx, DISTSIM_ERANGE, "cluster: alpha >= 2^40, beta >= 2^32, bucket >= 2^53 or more than 2^22 devices");
    if (C < 0) return fail(ctx, DISTSIM_EINVAL, "negative candidate count");
    if (C > 0x7fffffff) return fail(ctx, DISTSIM_ELIMIT, "candidate count outside [0, 2^31)");
    if (C != events->num_candidates) return fail(ctx, DISTSIM_EINVAL, "C differs from the distsim_build_events call");
    if (C == 0) return DISTSIM_OK;
    if (!batch_ns || !events->status || !events->num_events || !events->workspace || !cand_arrays_ok(cd) ||
        (events->stage_cap > 0 && (!comp_busy_ns || !comm_busy_ns)))
        return fail(ctx, DISTSIM_EINVAL, "null output, candidate or events array");
    if (events->L < 1 || events->L > DISTSIM_MAX_L || events->V < 1 || events->V > DISTSIM_MAX_V)
        return fail(ctx, DISTSIM_EINVAL, "events were not produced by distsim_build_events");
    Workspace ws;
    if (events->workspace_bytes < carve(ws, events->workspace, events->L, events->V, C))
        return fail(ctx, DISTSIM_EINVAL, "workspace too small for C");
    DeviceScope dev(ctx->device);
    HIP_TRY(dev.err);
    hipStream_t st = (hipStream_t)hip_stream;
    const CostsDev co = costs_after_build(events, ws);
    const CandDev ca = cand_dev(cd);
    const ClusterDev cl = to_dev(*cluster);
    EventsDev ev{events->stage_cap, events->status, events->stage_pos, events->stage_tab, events->stage_layers,
                 events->num_events};
    SimOut out{batch_ns, comp_busy_ns, comm_busy_ns, util};
    // k_sim_init marks the candidates that k_decode rejected; the sweeps write the others' results,
    // so that work may run beside them: for a long list k_simulate_gpipe does it on its way in
    const bool beside = cl.blocking != 2 && C >= ctx->split_min_items;
    if (!beside) {
        Timer t(ctx, st, DISTSIM_K_SIM_INIT);
        hipLaunchKernelGGL(k_sim_init, dim3((int)((C + 255) / 256)), dim3(256), 0, st, events->status, C, batch_ns);
    }
    // The sweep kernels below set EXEC by hand (DISTSIM_STEP*): blocks of kSimBlock threads, whole
    // wavefronts only, never a partial block.
    if (cl.blocking == 2) {
        Timer t(ctx, st, DISTSIM_K_SIMULATE);
        hipLaunchKernelGGL(k_simulate_links, dim3(simulate_grid(ctx, C) * (256 / kSimBlock)), dim3(kSimBlock), 0, st, co, cl, ca, ws, ev, out);
    } else if (C < ctx->split_min_items) {
        // a list of fewer candidates than that has fewer wave-items too: k_simulate takes all of it
        Timer t(ctx, st, DISTSIM_K_SIMULATE);
        hipLaunchKernelGGL(k_simulate, dim3(general_grid(ctx, C) * (256 / kSimBlock)), dim3(kSimBlock), 0, st, co, cl, ca, ws, ev, out);
    } else {
        // k_simulate and, for the pairs of GPipe items that it leaves out, k_simulate_gpipe, side
        // by side: they write different rows.  The timer of k_simulate spans both.
        Timer t(ctx, st, DISTSIM_K_SIMULATE);
        HIP_TRY(hipEventRecord(ctx->fork, st));
        HIP_TRY(hipStreamWaitEvent(ctx->side, ctx->fork, 0));
        hipLaunchKernelGGL(k_simulate, dim3(general_grid(ctx, C) * (256 / kSimBlock)), dim3(kSimBlock), 0, st, co, cl, ca, ws, ev, out);
        {
            // its first threads mark the rejected candidates (k_sim_init's work).  Its items all cost about
            // the same, so a wavefront may take several pairs in turn: a quarter of the wavefronts (measured:
            // span -1.5 %, and a quarter of the spill stores, which every wavefront makes once) -- unless the
            // all-reduce is bucketed: then an item's epilogue walks its layers with a trip to the tables
            // every few of them, and the launch needs the wavefronts to hide those (measured: +3 % with fewer)
            Timer tg(ctx, ctx->side, DISTSIM_K_SIMULATE_GPIPE);
            const int per_group = cl.bucket > 0 ? 256 / kSimBlock : 1;
            hipLaunchKernelGGL(k_simulate_gpipe, dim3(gpipe_grid(ctx, C) * per_group), dim3(kSimBlock), 0, ctx->side, co, cl, ca, ws, ev, out, C);
        }
        HIP_TRY(hipEventRecord(ctx->join, ctx->side));
        HIP_TRY(hipStreamWaitEvent(st, ctx->join, 0));
    }
    if (cd->chunks) {       // candidates of the interleaved schedule, if the caller has any
        // one launch for all classes; a block is one wavefront with 9.5 KB of LDS, 16 fit a CU; four
        // times as many blocks as fit, so that the order in which they start evens out their lengths
        Timer t(ctx, st, DISTSIM_K_SIMULATE_VIRTUAL);
        const int64_t most = (int64_t)ctx->num_cus * 64;
        const unsigned blocks = (unsigned)(C < most ? C : most);
        hipLaunchKernelGGL(k_simulate_virtual, dim3(blocks), dim3(kWave), 0, st, co, cl, ca, ws, ev, out);
    }
    if (cd->chunks && ca.n_schedules > 0) {       // candidates with an explicit schedule, if the caller has any
        Timer t(ctx, st, DISTSIM_K_SIMULATE_EXPLICIT);
        {
            // those whose schedule has a program: one launch for all classes, a block is one wavefront
            // with 12 KB of LDS; more blocks than fit, so that the order in which they start evens out their lengths
            const int64_t most = (int64_t)ctx->num_cus * 32;
            const unsigned blocks = (unsigned)(C < most ? C : most);
            hipLaunchKernelGGL(k_simulate_scheduled, dim3(blocks), dim3(kWave), 0, st, co, cl, ca, ws, ev, out);
        }
        // the others (none as a rule: every block ends at once then)
        const int64_t most = (int64_t)ctx->num_cus * 16;
        const unsigned blocks = (unsigned)(C < most ? C : most);
        hipLaunchKernelGGL(k_simulate_explicit, dim3(blocks), dim3(kWave), 0, st, co, cl, ca, ws, ev, out);
    }
    HIP_TRY(hipGetLastError());
    return DISTSIM_OK;
}

// Selection length from which the closed-form dump of the GPipe candidates runs beside the
// level-sweep dump on the context's stream; below it the fork and the join cost more than they bring.
static const int64_t kTimelineForkMin = 2048;

int distsim_timeline(distsim_ctx* ctx, const distsim_cluster* cluster, const distsim_candidates* cd,
                     const distsim_events* events, int64_t n, const int64_t* sel, const int64_t* task_off,
                     int64_t* start_ns, int64_t* end_ns, int64_t* ar_start_ns, int64_t* ar_end_ns, void* hip_stream) {
    if (!ctx) return DISTSIM_EINVAL;
    if (!cluster || !events || !cd) return fail(ctx, DISTSIM_EINVAL, "null argument");
    if (!cluster_ok(cluster)) return fail(ctx, DISTSIM_EINVAL, "cluster description out of range");
    if (!cluster_in_range(cluster)) return fail(ctx, DISTSIM_ERANGE, "cluster: alpha >= 2^40, beta >= 2^32, bucket >= 2^53 or more than 2^22 devices");
    if (n < 0) return fail(ctx, DISTSIM_EINVAL, "negative selection size");
    if (n > 0x7fffffff) return fail(ctx, DISTSIM_ELIMIT, "selection size outside [0, 2^31)");
    if (n == 0) return DISTSIM_OK;
    if (!sel || !task_off || !start_ns || !end_ns || !ar_start_ns || !ar_end_ns || !events->status ||
        !events->workspace || !cand_arrays_ok(cd))
        return fail(ctx, DISTSIM_EINVAL, "null array");
    if (events->L < 1 || events->L > DISTSIM_MAX_L || events->V < 1 || events->V > DISTSIM_MAX_V)
        return fail(ctx, DISTSIM_EINVAL, "events were not produced by distsim_build_events");
    Workspace ws;
    if (events->workspace_bytes < carve(ws, events->workspace, events->L, events->V, events->num_candidates))
        return fail(ctx, DISTSIM_EINVAL, "events were not produced by distsim_build_events");
    DeviceScope dev(ctx->device);
    HIP_TRY(dev.err);
    hipStream_t st = (hipStream_t)hip_stream;
    const CostsDev co = costs_after_build(events, ws);
    const CandDev ca = cand_dev(cd);
    {
        // k_timeline uses the DISTSIM_STEP* macros: blocks of one whole wavefront.  The selection is
        // packed into wave-items first (counting sort by width class); the sorted entry numbers and
        // the counters sit in workspace arrays that only distsim_build_events uses otherwise (the
        // ordering keys, one int32 per candidate, and the bin counters), so a selection longer than
        // the candidate list goes in several rounds.
        Timer t(ctx, st, DISTSIM_K_TIMELINE);
        const int64_t room = events->num_candidates > 0 ? events->num_candidates : 1;
        for (int64_t at = 0; at < n; at += room) {
            const int64_t nn = n - at < room ? n - at : room;
            const TimelineOut out{sel + at, task_off + at, start_ns, end_ns, ar_start_ns + at * kMaxPP, ar_end_ns + at * kMaxPP};
            const unsigned pb = (unsigned)((nn + 255) / 256);
            hipLaunchKernelGGL(k_timeline_clear, dim3(1), dim3(kWave), 0, st, ws.bin_count);
            hipLaunchKernelGGL(k_timeline_pack<0>, dim3(pb), dim3(256), 0, st, ca, events->status, events->num_candidates, nn,
                               out.sel, ws.bin_count, ws.key, out.ar_start, out.ar_end);
            // The dump of the GPipe candidates goes behind the first pack, which sets all all-reduce
            // windows to "none"; for a long selection on the context's stream, beside the second pack
            // and the level-sweep dump (they write different entries).
            const bool beside = nn >= kTimelineForkMin;
            const hipStream_t sg = beside ? ctx->side : st;
            auto dump_gpipe = [&]() {
                Timer tg(ctx, sg, DISTSIM_K_TIMELINE_GPIPE);
                hipLaunchKernelGGL(k_timeline_gpipe, dim3((unsigned)nn), dim3(kTlGpipeBlock), 0, sg, co, cl_dev(*cluster), ca, ws,
                                   events->status, events->num_candidates, nn, out);     // a workgroup per entry of the selection
            };
            if (beside) {
                HIP_TRY(hipEventRecord(ctx->fork, st));
                HIP_TRY(hipStreamWaitEvent(ctx->side, ctx->fork, 0));
                dump_gpipe();
            }
            hipLaunchKernelGGL(k_timeline_pack<1>, dim3(pb), dim3(256), 0, st, ca, events->status, events->num_candidates, nn,
                               out.sel, ws.bin_count, ws.key, out.ar_start, out.ar_end);
            hipLaunchKernelGGL(k_timeline, dim3((unsigned)nn), dim3(kWave), 0, st, co, cl_dev(*cluster), ca, ws,
                               events->status, events->num_candidates, nn, ws.bin_count, ws.key, out);
            if (beside) {
                HIP_TRY(hipEventRecord(ctx->join, ctx->side));
                HIP_TRY(hipStreamWaitEvent(st, ctx->join, 0));
            } else {
                dump_gpipe();
            }
        }
    }
    if (cd->chunks) {          // interleaved candidates among the selected ones: one wavefront each
        Timer t(ctx, st, DISTSIM_K_TIMELINE_VIRTUAL);
        const int64_t grid = n < 65536 ? n : 65536;
        hipLaunchKernelGGL(k_timeline_virtual, dim3((unsigned)grid), dim3(kWave), 0, st, co, cl_dev(*cluster), ca, ws,
                           events->status, events->num_candidates, n, sel, task_off, start_ns, end_ns, ar_start_ns,
                           ar_end_ns);
    }
    if (cd->chunks && ca.n_schedules > 0) {          // ... and those with an explicit schedule
        Timer t(ctx, st, DISTSIM_K_TIMELINE_EXPLICIT);
        const int64_t grid = n < 65536 ? n : 65536;
        hipLaunchKernelGGL(k_timeline_explicit, dim3((unsigned)grid), dim3(kWave), 0, st, co, cl_dev(*cluster), ca, ws,
                           events->status, events->num_candidates, n, sel, task_off, start_ns, end_ns, ar_start_ns,
                           ar_end_ns);
    }
    HIP_TRY(hipGetLastError());
    return DISTSIM_OK;
}

size_t distsim_search_scratch_bytes(int64_t C) {
    (void)C;
    return (size_t)kSearchMaxBlocks * sizeof(Best);
}

namespace {

// The two launches of the argmin; `partial` holds one Best per workgroup of the first.
int launch_search(distsim_ctx* ctx, const int64_t* batch_ns, const int64_t* weight, int64_t C, int objective,
                  int64_t* best, Best* partial, hipStream_t st) {
    int64_t nb = (C + kSearchBlock * 4 - 1) / (kSearchBlock * 4);
    if (nb > kSearchMaxBlocks) nb = kSearchMaxBlocks;
    if (nb < 1) nb = 1;
    if (objective == 0) {
        hipLaunchKernelGGL(k_search_partial<0>, dim3((int)nb), dim3(kSearchBlock), 0, st, batch_ns, weight, C, partial);
        hipLaunchKernelGGL(k_search_final<0>, dim3(1), dim3(kSearchBlock), 0, st, partial, (int)nb, best);
    } else {
        hipLaunchKernelGGL(k_search_partial<1>, dim3((int)nb), dim3(kSearchBlock), 0, st, batch_ns, weight, C, partial);
        hipLaunchKernelGGL(k_search_final<1>, dim3(1), dim3(kSearchBlock), 0, st, partial, (int)nb, best);
    }
    HIP_TRY(hipGetLastError());
    return DISTSIM_OK;
}

}  // namespace

int distsim_search(distsim_ctx* ctx, const int64_t* batch_ns, const int64_t* weight, int64_t C, int objective,
                   int64_t* best, void* scratch_mem, void* hip_stream) {
    if (!ctx) return DISTSIM_EINVAL;
    if (!best || !scratch_mem || (C > 0 && !batch_ns)) return fail(ctx, DISTSIM_EINVAL, "null argument");
    if (objective != 0 && objective != 1) return fail(ctx, DISTSIM_EINVAL, "objective must be 0 or 1");
    if (objective == 1 && C > 0 && !weight) return fail(ctx, DISTSIM_EINVAL, "objective 1 needs weights");
    if (C < 0) return fail(ctx, DISTSIM_EINVAL, "negative candidate count");
    DeviceScope dev(ctx->device);
    HIP_TRY(dev.err);
    hipStream_t st = (hipStream_t)hip_stream;
    Timer t(ctx, st, DISTSIM_K_SEARCH);
    return launch_search(ctx, batch_ns, weight, C, objective, best, (Best*)scratch_mem, st);
}

int distsim_search_static(distsim_ctx* ctx, const int64_t* batch_ns, const int64_t* weight, int64_t C, int objective,
                          int64_t* best, void* hip_stream) {
    if (!ctx) return DISTSIM_EINVAL;
    if (!best || (C > 0 && !batch_ns)) return fail(ctx, DISTSIM_EINVAL, "null argument");
    if (objective != 0 && objective != 1) return fail(ctx, DISTSIM_EINVAL, "objective must be 0 or 1");
    if (objective == 1 && C > 0 && !weight) return fail(ctx, DISTSIM_EINVAL, "objective 1 needs weights");
    if (C < 0) return fail(ctx, DISTSIM_EINVAL, "negative candidate count");
    if (C > DISTSIM_SEARCH_STATIC_MAX_C)
        return fail(ctx, DISTSIM_ELIMIT, "distsim_search_static: more than DISTSIM_SEARCH_STATIC_MAX_C (2^31 - 1) candidates");
    if (!ctx->static_scratch) return fail(ctx, DISTSIM_EHIP, ctx->static_scratch_err.empty() ? "no static scratch" : ctx->static_scratch_err);
    static_assert(sizeof(scratch) == DISTSIM_SEARCH_STATIC_SCRATCH_BYTES, "header and array disagree");
    DeviceScope dev(ctx->device);
    HIP_TRY(dev.err);
    // no timer here: its events would be created on first use, and this call creates nothing
    return launch_search(ctx, batch_ns, weight, C, objective, best, (Best*)ctx->static_scratch, (hipStream_t)hip_stream);
}

int distsim_bubbles(distsim_ctx* ctx, const distsim_candidates* cd, const distsim_events* events, int64_t n,
                    const int64_t* sel, const int64_t* task_off, const int64_t* start_ns, const int64_t* end_ns,
                    int64_t* idle_before_ns, void* hip_stream) {
    if (!ctx) return DISTSIM_EINVAL;
    if (!events || !cd) return fail(ctx, DISTSIM_EINVAL, "null argument");
    if (n < 0) return fail(ctx, DISTSIM_EINVAL, "negative selection size");
    if (n > 0x7fffffff) return fail(ctx, DISTSIM_ELIMIT, "selection size outside [0, 2^31)");
    if (n == 0) return DISTSIM_OK;
    if (!sel || !task_off || !start_ns || !end_ns || !idle_before_ns || !events->status || !cd->pp || !cd->m ||
        !cd->schedule)
        return fail(ctx, DISTSIM_EINVAL, "null array");
    DeviceScope dev(ctx->device);
    HIP_TRY(dev.err);
    hipStream_t st = (hipStream_t)hip_stream;
    const CandDev ca = cand_dev(cd);
    {
        Timer t(ctx, st, DISTSIM_K_BUBBLES);
        hipLaunchKernelGGL(k_bubbles, dim3((unsigned)n), dim3(256), 0, st, ca, events->status, events->num_candidates,
                           n, sel, task_off, start_ns, end_ns, idle_before_ns);
    }
    HIP_TRY(hipGetLastError());
    return DISTSIM_OK;
}

namespace {

struct DedupSpace {
    int64_t table_size;          // power of two >= 2n
    int32_t *table, *slot_of, *excl, *block_tot;
};

size_t carve_dedup(DedupSpace& d, void* base, int64_t n) {
    size_t off = 0;
    char* b = (char*)base;
    auto take = [&](size_t bytes) { void* p = b ? (void*)(b + off) : nullptr; off += align256(bytes); return p; };
    const int64_t nn = n > 0 ? n : 1;
    int64_t size = 64;
    while (size < 2 * nn) size <<= 1;
    d.table_size = size;
    d.table = (int32_t*)take((size_t)size * 4);
    d.slot_of = (int32_t*)take((size_t)nn * 4);
    d.excl = (int32_t*)take((size_t)nn * 4);
    d.block_tot = (int32_t*)take((size_t)((nn + kScanBlock - 1) / kScanBlock) * 4);
    return off;
}

constexpr int64_t kMaxDedupRecords = 1ll << 28;

}  // namespace

size_t distsim_dedup_workspace_bytes(int64_t n) {
    if (n < 0 || n > kMaxDedupRecords) return 0;
    DedupSpace d;
    return carve_dedup(d, nullptr, n);
}

int distsim_dedup_events(distsim_ctx* ctx, const int64_t* records, int64_t n, int32_t K, int32_t* event_id,
                         int32_t* rep, int64_t* num_events, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    if (!ctx) return DISTSIM_EINVAL;
    if (n < 0 || K < 1 || !num_events) return fail(ctx, DISTSIM_EINVAL, "bad size or null num_events");
    if (K > kMaxRecordWords || n > kMaxDedupRecords) return fail(ctx, DISTSIM_ELIMIT, "K above 16 or n above 2^28");
    if (n > 0 && (!records || !event_id || !rep || !workspace)) return fail(ctx, DISTSIM_EINVAL, "null argument");
    DedupSpace d;
    if (workspace_bytes < carve_dedup(d, workspace, n) && n > 0) return fail(ctx, DISTSIM_EINVAL, "workspace too small");
    DeviceScope dev(ctx->device);
    HIP_TRY(dev.err);
    hipStream_t st = (hipStream_t)hip_stream;
    Timer t(ctx, st, DISTSIM_K_DEDUP);
    const int64_t nb = (n + kScanBlock - 1) / kScanBlock;
    if (n > 0) {
        hipLaunchKernelGGL(k_dedup_clear, dim3((unsigned)((d.table_size + 255) / 256)), dim3(256), 0, st, d.table,
                           d.table_size);
        // dynamic LDS: the workgroup's records (K words of 8 B for each of its threads), for records of up to
        // kDedupStagedWords words; longer ones are compared through memory
        hipLaunchKernelGGL(k_dedup_insert, dim3((unsigned)((n + kDedupBlock - 1) / kDedupBlock)), dim3(kDedupBlock),
                           K <= kDedupStagedWords ? (size_t)K * kDedupBlock * sizeof(int64_t) : 0, st, records, n, (int)K,
                           d.table, d.table_size, d.slot_of);
        hipLaunchKernelGGL(k_dedup_scan_blocks, dim3((unsigned)nb), dim3(kScanBlock), 0, st, d.table, d.slot_of, n,
                           d.excl, d.block_tot);
    }
    hipLaunchKernelGGL(k_dedup_scan_totals, dim3(1), dim3(kScanBlock), 0, st, n > 0 ? d.block_tot : nullptr, nb,
                       num_events);
    if (n > 0)
        hipLaunchKernelGGL(k_dedup_assign, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d.table, d.slot_of,
                           d.excl, d.block_tot, n, event_id, rep);
    HIP_TRY(hipGetLastError());
    return DISTSIM_OK;
}

int distsim_comm_event_times(distsim_ctx* ctx, int64_t n, const int32_t* kind, const int32_t* ranks,
                             const int64_t* t_a, const int64_t* t_b, int64_t* elapsed_ns, void* hip_stream) {
    if (!ctx) return DISTSIM_EINVAL;
    if (n < 0) return fail(ctx, DISTSIM_EINVAL, "negative size");
    if (n == 0) return DISTSIM_OK;
    if (!kind || !ranks || !t_a || !t_b || !elapsed_ns) return fail(ctx, DISTSIM_EINVAL, "null argument");
    DeviceScope dev(ctx->device);
    HIP_TRY(dev.err);
    hipStream_t st = (hipStream_t)hip_stream;
    Timer t(ctx, st, DISTSIM_K_COMM_TIMES);
    hipLaunchKernelGGL(k_comm_event_times, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, n, kind, ranks, t_a,
                       t_b, elapsed_ns);
    HIP_TRY(hipGetLastError());
    return DISTSIM_OK;
}

int distsim_timing_enable(distsim_ctx* ctx, int on) {
    if (!ctx) return DISTSIM_EINVAL;
    ctx->timing = on != 0;
    return DISTSIM_OK;
}

int distsim_timing_read(distsim_ctx* ctx, int kernel, double* total_ms, int64_t* launches) {
    if (!ctx) return DISTSIM_EINVAL;
    if (kernel < 0 || kernel >= DISTSIM_K_COUNT || !total_ms || !launches)
        return fail(ctx, DISTSIM_EINVAL, "bad kernel id or null output");
    double tot = 0.0;
    int64_t n = 0;
    for (auto& tl : ctx->rec[kernel]) {
        HIP_TRY(hipEventSynchronize(tl.stop));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, tl.start, tl.stop));
        tot += ms;
        n++;
        ctx->pool.push_back(tl);
    }
    ctx->rec[kernel].clear();
    *total_ms = tot;
    *launches = n;
    return DISTSIM_OK;
}

const char* distsim_kernel_name(int kernel) {
    return kernel >= 0 && kernel < DISTSIM_K_COUNT ? kKernelNames[kernel] : "?";
}

}  // extern "C"
