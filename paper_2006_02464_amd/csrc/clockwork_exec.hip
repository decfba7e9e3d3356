// C ABI of the worker hot path (see include/clockwork_exec.h for the contract).
#include "../../include/clockwork_exec_introspect.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <functional>
#include <memory>
#include <mutex>
#include <string>
#include <vector>

#include "plan.h"

using namespace cw;

namespace {

constexpr int kMaxSlots = 64;
constexpr size_t kDefaultPageBytes = (size_t)16 << 20;  // the paper's page size (section 5.1)
constexpr int kProfileEvents = 128;  // EXECs timed back to back between two host syncs

enum SlotState { SLOT_FREE = 0, SLOT_INPUT, SLOT_EXECUTED };

struct Slot {
    SlotState state = SLOT_FREE;
    int32_t model = -1, batch = 0;
    size_t off = 0, bytes = 0;               // region in the IO cache
    size_t in_off = 0, logits_off = 0, probs_off = 0;
    hipEvent_t input_done = nullptr, exec_start = nullptr, exec_end = nullptr, released = nullptr;
    bool release_pending = false;            // `released` guards reuse of the region
};

// The slot-independent middle of a plan (everything between the input cast and the FC) as one
// executable HIP graph: kernel arguments only name workspace and weight-pool addresses, which
// are fixed once the weights are resident.
struct PlanGraph {
    hipGraphExec_t exec = nullptr;
    size_t first = 0, last = 0;  // launches [first, last] are inside the graph
};

// The graphs of a model's plans for one placement of its weights.  A model keeps the sets of the
// last few placements it had: coming back into pages it has been in before needs no recording,
// and no graph is destroyed while the worker runs unless a model moves through more than
// kMaxGraphSets placements (destroying one was measured at about a millisecond, during which other
// threads' launches stall).
struct GraphSet {
    std::vector<int32_t> pages;    // weight placement the graphs were captured for
    std::vector<PlanGraph> plans;  // parallel to m.plans
    uint64_t last_used = 0;        // LOAD counter value when it was last the active set
};
constexpr size_t kMaxGraphSets = 8;

struct ModelRt {
    Model m;
    bool loaded = false;
    std::vector<int32_t> pages;  // pool page of each of the model's weight pages while resident
    hipEvent_t load_done = nullptr;
    hipEvent_t last_exec_end = nullptr;  // end event of the last EXEC issued on these weights (a slot's event; not owned)
    std::vector<GraphSet> graph_sets;  // at most kMaxGraphSets
    int active_set = -1;               // the set recorded for `pages`, if there is one
    std::vector<std::vector<ResLayer>> res_programs;  // host copies of the resident programs uploaded by the last LOAD
};

}  // namespace

// ---- the arena of cw_exec_static: device memory that exists without an allocation --------------
// One array per GPU the library runs on, held until the process ends.  In host code the array's
// name is only a handle for the runtime; its device address on a GPU is asked for once, with that
// GPU current, and kept (every GPU has its own copy at its own address).
constexpr size_t kStaticScratchBytes = (size_t)80 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
char *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on `device`, which must be the current device.  Asked for once per
// device (cw_create does it); later calls only read the table.
hipError_t scratch_address(int device, char **out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<char *>(p);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}
}  // namespace

// A LOAD between its begin and its end: the placement it took and the graphs recorded for it.
struct cw_load_pending {
    int32_t model_id = -1;
    std::vector<int32_t> pages;     // the model's pages as the LOAD took them
    std::vector<char> want;         // per plan: record a graph for this placement
    std::vector<PlanGraph> graphs;  // recorded, then (after the end) the ones to destroy
    int32_t status = CW_OK;
    std::string err;
};

struct cw_ctx {
    int device = -1;       // -1: planning-only context without a GPU
    char *static_scratch = nullptr;  // this GPU's copy of `scratch`
    cw_config cfg{};
    char *workspace = nullptr, *io = nullptr, *pool = nullptr, *staging = nullptr;
    RangeAllocator io_alloc;
    size_t page_bytes = 0;            // weight pool page size
    std::vector<int32_t> free_pages;  // free pages of the weight pool, lowest index last (taken first)
    std::vector<hipEvent_t> page_guard;  // per page: end event of the last EXEC that may still read it (nullptr: none)
    Slot slots[kMaxSlots];
    std::vector<std::unique_ptr<ModelRt>> models;
    PlanOverride ov;
    hipStream_t internal_stream = nullptr;
    hipStream_t capture_stream = nullptr;  // only ever used to record graphs
    bool use_graphs = true;
    uint64_t load_counter = 0;             // orders the graph sets of a model by last use
    hipEvent_t staging_free = nullptr;  // last LOAD's pack kernels are done with the staging area
    bool staging_used = false;
    hipEvent_t prof_ev[2 * kProfileEvents] = {};
    // one EXEC at a time: remember where the last one went
    hipStream_t last_exec_stream = nullptr;
    hipEvent_t last_exec_end = nullptr;
    unsigned *res_error = nullptr;   // pinned host word a resident launch raises when it gives up (see kernels_resident.hip)
    bool resident_capable = true;    // 256 CUs in 8 XCDs (planning-only contexts: assumed)
    std::string err;
};

namespace {

int32_t set_err(cw_ctx *c, int32_t code, const std::string &msg) {
    if (c) c->err = msg;
    return code;
}

int32_t hip_fail(cw_ctx *c, hipError_t e, const char *what) {
    char buf[256];
    snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
    return set_err(c, CW_ERR_HIP, buf);
}

#define CW_HIP(ctx, call)                                   \
    do {                                                    \
        hipError_t e__ = (call);                            \
        if (e__ != hipSuccess) return hip_fail(ctx, e__, #call); \
    } while (0)

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(dev) == hipSuccess) ok = true;
    }
    ~DeviceGuard() {
        if (ok && prev >= 0) (void)hipSetDevice(prev);
    }
};

ModelRt *get_model(cw_ctx *c, int32_t id) {
    if (!c || id < 0 || id >= (int32_t)c->models.size()) return nullptr;
    return c->models[id].get();
}

Plan *get_plan(ModelRt *m, int32_t batch) {
    for (Plan &p : m->m.plans)
        if (p.batch == batch) return &p;
    return nullptr;
}

// Where the plan's address spaces are for one EXEC: the arena of intermediates and the three
// per-request buffers (the context's workspace and an IO slot, or the static scratch array and the
// caller's own device buffers).
struct Bases {
    char *workspace = nullptr, *input = nullptr, *logits = nullptr, *probs = nullptr;
    const int32_t *pages = nullptr;  // pool page of each of the model's weight pages
};

Bases bases_of(const cw_ctx *c, const ModelRt *m, const Slot *s) {
    Bases b;
    b.workspace = c->workspace;
    b.pages = m->pages.data();
    if (s) { b.input = c->io + s->in_off; b.logits = c->io + s->logits_off; b.probs = c->io + s->probs_off; }
    return b;
}

char *resolve(cw_ctx *c, const ModelRt *m, const Bases &b, const Ref &r) {
    switch (r.space) {
        case SP_WORKSPACE: return b.workspace + r.offset;
        case SP_WEIGHTS: return c->pool + (size_t)b.pages[r.offset / c->page_bytes] * c->page_bytes + r.offset % c->page_bytes;
        case SP_SLOT_INPUT: return b.input;
        case SP_SLOT_LOGITS: return b.logits;
        case SP_SLOT_PROBS: return b.probs;
        default: return nullptr;
    }
}

hipError_t issue(cw_ctx *c, const ModelRt *m, const Bases &s, const Launch &l, hipStream_t st) {
    const DType dt = m->m.dtype;
    switch (l.kind) {
        case K_CAST_INPUT: {
            CastArgs a = l.cast;
            a.x = reinterpret_cast<const float *>(resolve(c, m, s, l.x));
            a.y = resolve(c, m, s, l.y);
            return launch_cast_input(dt, a, st);
        }
        case K_CONV: {
            ConvArgs a = l.conv;
            a.x = resolve(c, m, s, l.x);
            a.w = resolve(c, m, s, l.w);
            a.bias = reinterpret_cast<const float *>(resolve(c, m, s, l.bias));
            a.res = resolve(c, m, s, l.res);
            a.y = resolve(c, m, s, l.y);
            a.partial = reinterpret_cast<float *>(resolve(c, m, s, l.partial));
            a.counters = reinterpret_cast<int32_t *>(resolve(c, m, s, l.counters));
            if (l.fused_bm > 0) {
                a.w2 = resolve(c, m, s, l.w2);
                a.bias2 = reinterpret_cast<const float *>(resolve(c, m, s, l.bias2));
                a.x2 = resolve(c, m, s, l.x2);
                a.wd = resolve(c, m, s, l.wd);
                a.biasd = reinterpret_cast<const float *>(resolve(c, m, s, l.biasd));
                a.w3 = resolve(c, m, s, l.w3);
                a.bias3 = reinterpret_cast<const float *>(resolve(c, m, s, l.bias3));
                a.y3 = resolve(c, m, s, l.y3);
                return launch_conv_fused(dt, l.fused_bm, l.fused_kg, a, st);
            }
            if (l.pair_op >= 0) {
                ConvArgs a0 = l.conv0;
                a0.x = a.x;
                a0.w = resolve(c, m, s, l.w0);
                a0.bias = reinterpret_cast<const float *>(resolve(c, m, s, l.bias0));
                a0.res = resolve(c, m, s, l.res0);
                a0.y = resolve(c, m, s, l.y0);
                return launch_conv_pair(dt, l.tile, a0, a, st);
            }
            return launch_conv(dt, l.tile, l.stem, a, st);
        }
        case K_MAXPOOL:
        case K_GAVGPOOL: {
            PoolArgs a = l.pool;
            a.x = resolve(c, m, s, l.x);
            a.y = resolve(c, m, s, l.y);
            if (l.kind == K_MAXPOOL && l.pool_bm > 0) {   // with the 1x1 convolution over the pooled tile
                ConvArgs cv = l.conv;
                cv.w = resolve(c, m, s, l.w);
                cv.bias = reinterpret_cast<const float *>(resolve(c, m, s, l.bias));
                cv.y = resolve(c, m, s, l.y2);
                return launch_maxpool_conv(dt, a, cv, l.pool_bm, st);
            }
            return l.kind == K_MAXPOOL ? launch_maxpool(dt, a, st) : launch_gavgpool(dt, a, st);
        }
        case K_FC: {
            FcArgs a = l.fc;
            a.f = reinterpret_cast<const float *>(resolve(c, m, s, l.x));
            a.w = resolve(c, m, s, l.w);
            a.bias = reinterpret_cast<const float *>(resolve(c, m, s, l.bias));
            a.z = reinterpret_cast<float *>(resolve(c, m, s, l.y));
            if (l.probs.space == SP_SLOT_PROBS) {
                a.p = reinterpret_cast<float *>(resolve(c, m, s, l.probs));
                a.partial = reinterpret_cast<float *>(resolve(c, m, s, l.partial));
                a.counters = reinterpret_cast<int32_t *>(resolve(c, m, s, l.counters));
            }
            return launch_fc(dt, a, st);
        }
        case K_SOFTMAX: {
            SoftmaxArgs a = l.sm;
            a.z = reinterpret_cast<const float *>(resolve(c, m, s, l.x));
            a.p = reinterpret_cast<float *>(resolve(c, m, s, l.y));
            return launch_softmax(a, st);
        }
        case K_DWCONV: {
            DwArgs a = l.dw;
            a.x = resolve(c, m, s, l.x);
            a.w = resolve(c, m, s, l.w);
            a.bias = reinterpret_cast<const float *>(resolve(c, m, s, l.bias));
            if (l.dw_fused) {   // with the 1x1 convolution over its result: res and y are that convolution's
                ConvArgs cv = l.conv;
                cv.w = resolve(c, m, s, l.w2);
                cv.bias = reinterpret_cast<const float *>(resolve(c, m, s, l.bias2));
                cv.res = resolve(c, m, s, l.res);
                cv.y = resolve(c, m, s, l.y);
                return launch_dwconv_conv(dt, a, cv, st);
            }
            a.res = resolve(c, m, s, l.res);
            a.y = resolve(c, m, s, l.y);
            return launch_dwconv(dt, a, st);
        }
        case K_RESIDENT: {
            ResidentArgs a{};
            a.layers = reinterpret_cast<const ResLayer *>(resolve(c, m, s, l.w));
            a.n_layers = (int32_t)l.members.size();
            a.workspace = s.workspace;
            a.flags = reinterpret_cast<unsigned *>(s.workspace + kCounterBytes + kResidentFlagsOff);
            a.flags_per_part = l.res_flags_per_part;
            a.epoch = reinterpret_cast<unsigned *>(s.workspace + kCounterBytes);
            a.error = c->res_error;
            a.spin_limit = 1u << 20;   // about a second of polling before a wait gives up
            return launch_resident(dt, a, st);
        }
        case K_WINO_INPUT:
        case K_WINO_OUTPUT: {
            WinoArgs a = l.wino;
            a.x = resolve(c, m, s, l.x);
            a.y = resolve(c, m, s, l.y);
            a.bias = reinterpret_cast<const float *>(resolve(c, m, s, l.bias));
            a.res = resolve(c, m, s, l.res);
            return l.kind == K_WINO_INPUT ? launch_wino_input(dt, a, st) : launch_wino_output(dt, a, st);
        }
        case K_COPY_CHANNELS: {
            CopyArgs a = l.copy;
            a.src = resolve(c, m, s, l.x);
            a.dst = resolve(c, m, s, l.y);
            return launch_copy_channels(a, st);
        }
    }
    return hipErrorInvalidValue;
}

// Checks shared by cw_exec and its instrumented twin.
int32_t exec_checks(cw_ctx *c, int32_t model_id, int32_t batch, int32_t slot, ModelRt **mo, Plan **po, Slot **so) {
    if (!c) return CW_ERR_INVALID;
    if (c->device < 0) return set_err(c, CW_ERR_INVALID, "planning-only context has no device");
    ModelRt *m = get_model(c, model_id);
    if (!m) return set_err(c, CW_ERR_INVALID, "unknown model id");
    Plan *p = get_plan(m, batch);
    if (!p) return set_err(c, CW_ERR_BAD_BATCH, "no plan for this batch size");
    if (!m->loaded) return set_err(c, CW_ERR_NOT_LOADED, "weights are not resident");
    if (slot < 0 || slot >= kMaxSlots || c->slots[slot].state == SLOT_FREE)
        return set_err(c, CW_ERR_NO_INPUT, "slot holds no input");
    Slot *s = &c->slots[slot];
    if (s->model != model_id) return set_err(c, CW_ERR_NO_INPUT, "slot holds an input for another model");
    if (s->batch != batch) return set_err(c, CW_ERR_BAD_BATCH, "slot holds an input of another batch size");
    *mo = m; *po = p; *so = s;
    return CW_OK;
}

int32_t exec_gate(cw_ctx *c, ModelRt *m, Slot *s, hipStream_t st) {
    if (c->last_exec_end && c->last_exec_stream != st) {
        hipError_t q = hipEventQuery(c->last_exec_end);
        if (q == hipErrorNotReady) return set_err(c, CW_ERR_BUSY, "an EXEC is in flight on another stream");
        if (q != hipSuccess) return hip_fail(c, q, "hipEventQuery");
    }
    CW_HIP(c, hipStreamWaitEvent(st, s->input_done, 0));
    CW_HIP(c, hipStreamWaitEvent(st, m->load_done, 0));
    return CW_OK;
}

void percentile_profile(std::vector<float> v, cw_profile *out) {
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    auto rank = [&](double q) {  // nearest rank
        size_t k = (size_t)std::ceil(q * (double)n);
        if (k < 1) k = 1;
        if (k > n) k = n;
        return v[k - 1];
    };
    out->n = (uint32_t)n;
    out->p50_us = rank(0.50);
    out->p99_us = rank(0.99);
    out->p999_us = rank(0.999);
    out->p9999_us = rank(0.9999);
    out->min_us = v.front();
    out->max_us = v.back();
    double s = 0;
    for (float x : v) s += x;
    out->mean_us = (float)(s / (double)n);
}

int32_t acquire_slot(cw_ctx *c, ModelRt *m, int32_t model_id, int32_t batch, hipStream_t st, int32_t *slot_out) {
    int idx = -1;
    for (int i = 0; i < kMaxSlots; ++i)
        if (c->slots[i].state == SLOT_FREE) { idx = i; break; }
    if (idx < 0) return set_err(c, CW_ERR_NO_SLOT, "every IO slot is in use");
    Slot &s = c->slots[idx];
    const size_t in_b = (size_t)batch * m->m.in_c * m->m.in_h * m->m.in_w * 4;
    const size_t out_b = (size_t)batch * m->m.classes * 4;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    const size_t total = up(in_b) + 2 * up(out_b);
    size_t off = 0;
    if (!c->io_alloc.alloc(total, &off)) return set_err(c, CW_ERR_NO_MEMORY, "IO cache is full");
    // The region may have belonged to a slot whose OUTPUT copies are still in flight: every
    // pending release is waited for by the stream that is about to overwrite IO memory.
    for (int i = 0; i < kMaxSlots; ++i) {
        Slot &o = c->slots[i];
        if (o.release_pending) {
            hipError_t q = hipEventQuery(o.released);
            if (q == hipErrorNotReady) {
                hipError_t e = hipStreamWaitEvent(st, o.released, 0);
                if (e != hipSuccess) { c->io_alloc.free(off, total); return hip_fail(c, e, "hipStreamWaitEvent"); }
            } else {
                o.release_pending = false;
            }
        }
    }
    s.state = SLOT_INPUT;
    s.model = model_id; s.batch = batch;
    s.off = off; s.bytes = total;
    s.in_off = off;
    s.logits_off = off + up(in_b);
    s.probs_off = s.logits_off + up(out_b);
    *slot_out = idx;
    return CW_OK;
}

void free_slot(cw_ctx *c, Slot *s) {
    if (s->state == SLOT_FREE) return;
    c->io_alloc.free(s->off, s->bytes);
    s->state = SLOT_FREE;
    s->model = -1;
}


bool slot_free(const Launch &l) {
    for (const Ref *r : {&l.x, &l.w, &l.bias, &l.res, &l.y, &l.partial, &l.counters, &l.probs, &l.y3})
        if (r->space == SP_SLOT_INPUT || r->space == SP_SLOT_LOGITS || r->space == SP_SLOT_PROBS) return false;
    return true;
}

void destroy_graphs(std::vector<PlanGraph> &graphs) {
    for (PlanGraph &g : graphs)
        if (g.exec) { (void)hipGraphExecDestroy(g.exec); g.exec = nullptr; }
}

// Records the slot-independent run of launches of every plan for which `want[pi]` is set into a
// graph whose kernel arguments hold the weight addresses of the placement `pages`.  Host work only:
// nothing executes.  Reads the context's constants, the model's plans (fixed once it is defined)
// and its own arguments, nothing else: it may run beside other calls on the same context, one
// recording at a time (there is one capture stream).
int32_t record_graphs(cw_ctx *c, const ModelRt *m, const std::vector<int32_t> &pages, const std::vector<char> &want,
                      std::vector<PlanGraph> *out, std::string *err) {
    out->clear();
    out->resize(m->m.plans.size());
    Bases b;
    b.workspace = c->workspace;
    b.pages = pages.data();
    auto fail = [&](hipError_t e, const char *what) {
        *err = std::string(what) + ": " + hipGetErrorString(e);
        return CW_ERR_HIP;
    };
    for (size_t pi = 0; pi < m->m.plans.size(); ++pi) {
        if (!want[pi]) continue;
        const Plan &p = m->m.plans[pi];
        PlanGraph &pg = (*out)[pi];
        // longest run of slot-independent launches
        size_t best_a = 0, best_n = 0, a = 0;
        for (size_t i = 0; i <= p.launches.size(); ++i) {
            if (i == p.launches.size() || !slot_free(p.launches[i])) {
                if (i - a > best_n) { best_n = i - a; best_a = a; }
                a = i + 1;
            }
        }
        if (best_n < 2) continue;
        hipGraph_t graph = nullptr;
        hipError_t e = hipStreamBeginCapture(c->capture_stream, hipStreamCaptureModeThreadLocal);
        if (e != hipSuccess) return fail(e, "hipStreamBeginCapture");
        for (size_t i = best_a; i < best_a + best_n && e == hipSuccess; ++i) e = issue(c, m, b, p.launches[i], c->capture_stream);
        hipError_t e2 = hipStreamEndCapture(c->capture_stream, &graph);
        if (e != hipSuccess || e2 != hipSuccess) {
            if (graph) (void)hipGraphDestroy(graph);
            return fail(e != hipSuccess ? e : e2, "graph capture");
        }
        e = hipGraphInstantiate(&pg.exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (e != hipSuccess) { pg.exec = nullptr; return fail(e, "hipGraphInstantiate"); }
        pg.first = best_a;
        pg.last = best_a + best_n - 1;
    }
    return CW_OK;
}

// Enqueues the launches of a plan: the recorded graph for its middle part when there is one.
int32_t enqueue_plan(cw_ctx *c, ModelRt *m, const Plan *p, const Slot *s, hipStream_t st) {
    const size_t pi = (size_t)(p - m->m.plans.data());
    // a graph holds the weight addresses of the placement it was recorded for: replay it only there
    const GraphSet *gs = (c->use_graphs && m->active_set >= 0) ? &m->graph_sets[m->active_set] : nullptr;
    const PlanGraph *pg = (gs && pi < gs->plans.size() && gs->plans[pi].exec) ? &gs->plans[pi] : nullptr;
    for (size_t i = 0; i < p->launches.size(); ++i) {
        if (pg && i == pg->first) {
            CW_HIP(c, hipGraphLaunch(pg->exec, st));
            i = pg->last;
            continue;
        }
        hipError_t e = issue(c, m, bases_of(c, m, s), p->launches[i], st);
        if (e != hipSuccess) return hip_fail(c, e, p->launches[i].info.name);
    }
    return CW_OK;
}

}  // namespace

extern "C" {

const char *cw_strerror(int32_t st) {
    switch (st) {
        case CW_OK: return "ok";
        case CW_ERR_INVALID: return "invalid argument";
        case CW_ERR_HIP: return "HIP runtime error";
        case CW_ERR_NO_MEMORY: return "pre-allocated pool exhausted";
        case CW_ERR_NOT_LOADED: return "weights not loaded";
        case CW_ERR_ALREADY_LOADED: return "weights already loaded";
        case CW_ERR_NO_INPUT: return "slot holds no input or result";
        case CW_ERR_BAD_BATCH: return "no plan for this batch size";
        case CW_ERR_BUSY: return "an EXEC is already in flight";
        case CW_ERR_UNSUPPORTED: return "unsupported topology or request";
        case CW_ERR_NO_SLOT: return "no free IO slot";
        case CW_ERR_TOO_LATE: return "action reached after its latest start time";
        case CW_ERR_TIMEOUT: return "timed out";
        default: return "unknown status";
    }
}

int32_t cw_context_device(cw_ctx *c) { return c ? c->device : -1; }

static thread_local std::string g_create_err;  // detail of a failed cw_create (no context yet)
const char *cw_last_error(cw_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

int32_t cw_create(cw_ctx **out, const cw_config *cfg) {
    if (!out || !cfg) return CW_ERR_INVALID;
    *out = nullptr;
    std::unique_ptr<cw_ctx> c(new cw_ctx);
    c->cfg = *cfg;
    c->device = cfg->device;
    c->io_alloc.reset(cfg->io_bytes);
    c->page_bytes = cfg->weight_page_bytes ? cfg->weight_page_bytes : kDefaultPageBytes;
    if (c->page_bytes % 256 != 0) { g_create_err = "weight_page_bytes must be a multiple of 256"; return CW_ERR_INVALID; }
    for (int32_t pg = (int32_t)(cfg->weight_pool_bytes / c->page_bytes) - 1; pg >= 0; --pg) c->free_pages.push_back(pg);
    c->page_guard.assign(c->free_pages.size(), nullptr);
    if (cfg->device < 0) {  // planning-only: models and plans can be defined and inspected
        *out = c.release();
        return CW_OK;
    }
    auto create_fail = [&](int32_t code, const char *what, hipError_t e) {
        g_create_err = std::string(what) + ": " + hipGetErrorString(e);
        return code;
    };
    int ndev = 0;
    hipError_t ce = hipGetDeviceCount(&ndev);
    if (ce != hipSuccess) return create_fail(CW_ERR_HIP, "hipGetDeviceCount", ce);
    if (cfg->device >= ndev) return create_fail(CW_ERR_INVALID, "device ordinal out of range", hipErrorInvalidDevice);
    DeviceGuard g(cfg->device);
    if (!g.ok) return create_fail(CW_ERR_HIP, "hipSetDevice", hipGetLastError());
    hipDeviceProp_t prop;
    if ((ce = hipGetDeviceProperties(&prop, cfg->device)) != hipSuccess) return create_fail(CW_ERR_HIP, "hipGetDeviceProperties", ce);
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)  // kernels exist for gfx950 only
        return create_fail(CW_ERR_UNSUPPORTED, prop.gcnArchName, hipErrorNoBinaryForGpu);
    cw_ctx *p = c.get();
    auto cleanup = [&]() { cw_destroy(c.release()); };
    auto dmalloc = [&](char **ptr, size_t bytes) {
        return bytes == 0 ? hipSuccess : hipMalloc(reinterpret_cast<void **>(ptr), bytes);
    };
    if (dmalloc(&p->workspace, cfg->workspace_bytes) != hipSuccess || dmalloc(&p->io, cfg->io_bytes) != hipSuccess ||
        dmalloc(&p->pool, cfg->weight_pool_bytes) != hipSuccess ||
        dmalloc(&p->staging, cfg->load_staging_bytes) != hipSuccess) {
        g_create_err = std::string("hipMalloc of the pools: ") + hipGetErrorString(hipGetLastError());
        cleanup();
        return CW_ERR_NO_MEMORY;
    }
    // split-K arrival counters must start at zero; every launch leaves them at zero again
    if (cfg->workspace_bytes < kCounterBytes + kResidentBytes || hipMemset(p->workspace, 0, kCounterBytes + kResidentBytes) != hipSuccess) {
        g_create_err = "workspace smaller than its header (split-K counters, resident-launch flags), or hipMemset failed";
        cleanup();
        return CW_ERR_NO_MEMORY;
    }
    if ((ce = scratch_address(cfg->device, &p->static_scratch)) != hipSuccess) {
        g_create_err = std::string("hipGetSymbolAddress of the static arena: ") + hipGetErrorString(ce);
        cleanup();
        return CW_ERR_HIP;
    }
    p->resident_capable = prop.multiProcessorCount == kResPartitions * kResGroupsPerPartition;
    if (hipHostMalloc(reinterpret_cast<void **>(&p->res_error), 64, hipHostMallocDefault) != hipSuccess) {
        g_create_err = "hipHostMalloc of the resident-launch error word failed";
        cleanup();
        return CW_ERR_HIP;
    }
    *p->res_error = 0u;
    bool ok = hipStreamCreateWithFlags(&p->internal_stream, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&p->capture_stream, hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&p->staging_free, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; ok && i < kMaxSlots; ++i) {
        Slot &s = p->slots[i];
        ok = hipEventCreateWithFlags(&s.input_done, hipEventDisableTiming) == hipSuccess &&
             hipEventCreate(&s.exec_start) == hipSuccess && hipEventCreate(&s.exec_end) == hipSuccess &&
             hipEventCreateWithFlags(&s.released, hipEventDisableTiming) == hipSuccess;
    }
    for (int i = 0; ok && i < 2 * kProfileEvents; ++i) ok = hipEventCreate(&p->prof_ev[i]) == hipSuccess;
    if (!ok) {
        g_create_err = std::string("stream/event creation: ") + hipGetErrorString(hipGetLastError());
        cleanup();
        return CW_ERR_HIP;
    }
    *out = c.release();
    return CW_OK;
}

int32_t cw_destroy(cw_ctx *c) {
    if (!c) return CW_ERR_INVALID;
    if (c->device >= 0) {
        DeviceGuard g(c->device);
        (void)hipDeviceSynchronize();
        for (auto &m : c->models) {
            if (m)
                for (GraphSet &gs : m->graph_sets) destroy_graphs(gs.plans);
            if (m && m->load_done) (void)hipEventDestroy(m->load_done);
        }
        if (c->capture_stream) (void)hipStreamDestroy(c->capture_stream);
        for (Slot &s : c->slots) {
            if (s.input_done) (void)hipEventDestroy(s.input_done);
            if (s.exec_start) (void)hipEventDestroy(s.exec_start);
            if (s.exec_end) (void)hipEventDestroy(s.exec_end);
            if (s.released) (void)hipEventDestroy(s.released);
        }
        for (hipEvent_t e : c->prof_ev)
            if (e) (void)hipEventDestroy(e);
        if (c->staging_free) (void)hipEventDestroy(c->staging_free);
        if (c->internal_stream) (void)hipStreamDestroy(c->internal_stream);
        if (c->res_error) (void)hipHostFree(c->res_error);
        if (c->workspace) (void)hipFree(c->workspace);
        if (c->io) (void)hipFree(c->io);
        if (c->pool) (void)hipFree(c->pool);
        if (c->staging) (void)hipFree(c->staging);
    }
    delete c;
    return CW_OK;
}

int32_t cw_set_debug_keep(cw_ctx *c, int32_t keep) {
    if (!c) return CW_ERR_INVALID;
    c->ov.keep_all = keep != 0;
    return CW_OK;
}

int32_t cw_set_plan_override(cw_ctx *c, int32_t conv_tile, int32_t split_k) {
    if (!c) return CW_ERR_INVALID;
    if (conv_tile >= (int32_t)N_CONV_TILES || split_k < 0) return set_err(c, CW_ERR_INVALID, "bad override");
    c->ov.tile = conv_tile < 0 ? -1 : conv_tile;
    c->ov.split_k = split_k;
    return CW_OK;
}

int32_t cw_set_fusion(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    if (on < 0 || on > 2) return set_err(c, CW_ERR_INVALID, "fusion mode must be 0, 1 or 2");
    c->ov.fuse = on;
    return CW_OK;
}

int32_t cw_set_fusion_third(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    if (on < 0 || on > 2) return set_err(c, CW_ERR_INVALID, "mode must be 0, 1 or 2");
    c->ov.fuse_third = on;
    return CW_OK;
}

int32_t cw_set_fusion_pool(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    c->ov.fuse_pool = on != 0;
    return CW_OK;
}

int32_t cw_set_fusion_dw(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    c->ov.fuse_dw = on != 0;
    return CW_OK;
}

int32_t cw_set_fc_softmax(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    c->ov.fc_softmax = on != 0;
    return CW_OK;
}

int32_t cw_set_panels(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    c->ov.panels = on != 0;
    return CW_OK;
}

int32_t cw_set_resident(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    if (on && !c->resident_capable) return set_err(c, CW_ERR_UNSUPPORTED, "resident launches need 256 compute units in 8 XCDs");
    if (on < 0 || on > 2) return set_err(c, CW_ERR_INVALID, "resident mode must be 0, 1 or 2");
    c->ov.resident = on;
    return CW_OK;
}

int32_t cw_set_winograd(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    c->ov.winograd = on != 0;
    return CW_OK;
}

int32_t cw_set_pair_launches(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    c->ov.pair = on != 0;
    return CW_OK;
}

int32_t cw_set_plan_table(cw_ctx *c, const int32_t *rows, int32_t n_rows) {
    if (!c || n_rows < 0 || (n_rows > 0 && !rows)) return set_err(c, CW_ERR_INVALID, "null table");
    std::vector<TunedShape> t;
    for (int32_t i = 0; i < n_rows; ++i) {
        const int32_t *r = rows + 7 * i;
        if (r[5] < 0 || r[5] >= (int32_t)N_CONV_TILES || r[6] < 1) return set_err(c, CW_ERR_INVALID, "bad tile or split-K in a table row");
        t.push_back(TunedShape{r[0], r[1], r[2], r[3], r[4], r[5], r[6]});
    }
    c->ov.table.swap(t);
    return CW_OK;
}

int32_t cw_model_define(cw_ctx *c, const cw_op *ops, int32_t n_ops, int32_t in_c, int32_t in_h, int32_t in_w,
                        const int32_t *batch_sizes, int32_t n_batch, int32_t dtype, int32_t *model_id) {
    if (!c || !ops || !batch_sizes || n_batch < 1 || !model_id) return set_err(c, CW_ERR_INVALID, "null or empty argument");
    std::unique_ptr<ModelRt> m(new ModelRt);
    std::string err;
    int32_t rc = model_init(&m->m, ops, n_ops, in_c, in_h, in_w, dtype, c->page_bytes, c->ov.winograd, &err);
    if (rc != CW_OK) return set_err(c, rc, err);
    m->m.keep_all = c->ov.keep_all;
    for (int i = 0; i < n_batch; ++i) {
        if (get_plan(m.get(), batch_sizes[i])) continue;  // duplicate batch size
        Plan p;
        rc = plan_build(m->m, batch_sizes[i], c->ov, &p, &err);
        if (rc != CW_OK) return set_err(c, rc, err);
        if (p.workspace_bytes > c->cfg.workspace_bytes && c->device >= 0)
            return set_err(c, CW_ERR_NO_MEMORY, "plan needs more workspace than the context has");
        m->m.plans.push_back(std::move(p));
    }
    // resident programs live beside the model's packed weights (written at LOAD, when the weights'
    // addresses are known)
    for (Plan &p : m->m.plans)
        for (Launch &l : p.launches)
            if (l.kind == K_RESIDENT) {
                const size_t bytes = l.members.size() * sizeof(ResLayer);
                if (bytes > m->m.page_bytes) return set_err(c, CW_ERR_UNSUPPORTED, "a resident program is larger than a weight page");
                l.w = Ref{SP_WEIGHTS, model_reserve(&m->m, bytes)};
            }
    if (c->device >= 0) {
        DeviceGuard g(c->device);
        CW_HIP(c, hipEventCreateWithFlags(&m->load_done, hipEventDisableTiming));
    }
    c->models.push_back(std::move(m));
    *model_id = (int32_t)c->models.size() - 1;
    return CW_OK;
}

int32_t cw_model_define_resnet(cw_ctx *c, int32_t depth, int32_t in_h, int32_t in_w, int32_t dtype, int32_t *model_id) {
    if (!c) return CW_ERR_INVALID;
    std::vector<cw_op> ops;
    if (!resnet_ops(depth, &ops)) return set_err(c, CW_ERR_UNSUPPORTED, "depth must be 18, 50 or 152");
    static const int32_t batches[5] = {1, 2, 4, 8, 16};
    return cw_model_define(c, ops.data(), (int32_t)ops.size(), 3, in_h, in_w, batches, 5, dtype, model_id);
}

int32_t cw_model_get_ops(cw_ctx *c, int32_t model_id, cw_op *ops_out, int32_t cap, int32_t *n_ops) {
    ModelRt *m = get_model(c, model_id);
    if (!m || !n_ops) return set_err(c, CW_ERR_INVALID, "unknown model id");
    *n_ops = (int32_t)m->m.ops.size();
    if (ops_out)
        for (int i = 0; i < std::min(cap, *n_ops); ++i) ops_out[i] = m->m.ops[i];
    return CW_OK;
}

size_t cw_model_weight_bytes(cw_ctx *c, int32_t model_id) {
    ModelRt *m = get_model(c, model_id);
    return m ? m->m.blob_bytes : 0;
}

size_t cw_model_workspace_bytes(cw_ctx *c, int32_t model_id, int32_t batch) {
    ModelRt *m = get_model(c, model_id);
    Plan *p = m ? get_plan(m, batch) : nullptr;
    return p ? p->workspace_bytes : 0;
}

size_t cw_weight_pool_free(cw_ctx *c) { return c ? c->free_pages.size() * c->page_bytes : 0; }
int32_t cw_weight_pages_free(cw_ctx *c) { return c ? (int32_t)c->free_pages.size() : CW_ERR_INVALID; }
int32_t cw_model_weight_pages(cw_ctx *c, int32_t model_id) {
    ModelRt *m = c ? get_model(c, model_id) : nullptr;
    return m ? m->m.n_pages : CW_ERR_INVALID;
}

// Returns a model's pages to the pool; the free list stays sorted so that the lowest page is
// taken first and placement is a function of the LOAD/UNLOAD history alone.
static void release_pages(cw_ctx *c, ModelRt *m) {
    // An EXEC that reads these pages may still be queued or running: whoever writes them next waits
    // for its end event (UNLOAD itself stays metadata only).
    for (int32_t pg : m->pages) c->page_guard[pg] = m->last_exec_end;
    m->last_exec_end = nullptr;
    c->free_pages.insert(c->free_pages.end(), m->pages.begin(), m->pages.end());
    std::sort(c->free_pages.begin(), c->free_pages.end(), std::greater<int32_t>());
    m->pages.clear();
    m->active_set = -1;
}

int32_t cw_load_weights_begin(cw_ctx *c, int32_t model_id, const void *host_blob, size_t bytes, void *stream, cw_load_pending **pending) {
    if (!c || !pending) return CW_ERR_INVALID;
    *pending = nullptr;
    if (c->device < 0) return set_err(c, CW_ERR_INVALID, "planning-only context has no device");
    ModelRt *m = get_model(c, model_id);
    if (!m || !host_blob) return set_err(c, CW_ERR_INVALID, "unknown model id or null blob");
    if (bytes != m->m.blob_bytes) return set_err(c, CW_ERR_INVALID, "blob size does not match the model");
    if (m->loaded) return set_err(c, CW_ERR_ALREADY_LOADED, "model is resident");
    if (bytes > c->cfg.load_staging_bytes) return set_err(c, CW_ERR_NO_MEMORY, "blob larger than the LOAD staging area");
    // LOAD takes whole pages, any that are free (paper section 5.1): no fragmentation, and whether a
    // LOAD fits depends on the free-page count alone.
    if ((size_t)m->m.n_pages > c->free_pages.size()) return set_err(c, CW_ERR_NO_MEMORY, "not enough free weight pages");
    m->pages.assign(c->free_pages.end() - m->m.n_pages, c->free_pages.end());
    std::reverse(m->pages.begin(), m->pages.end());  // lowest page first
    c->free_pages.resize(c->free_pages.size() - m->m.n_pages);
    DeviceGuard g(c->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    auto bail = [&](hipError_t e, const char *what) {
        release_pages(c, m);
        return hip_fail(c, e, what);
    };
    hipError_t e;
    // One staging area: a LOAD waits for the previous LOAD's pack kernels.
    if (c->staging_used && (e = hipStreamWaitEvent(st, c->staging_free, 0)) != hipSuccess) return bail(e, "hipStreamWaitEvent");
    if ((e = hipMemcpyAsync(c->staging, host_blob, bytes, hipMemcpyHostToDevice, st)) != hipSuccess) return bail(e, "hipMemcpyAsync");
    // The pages may have belonged to a model whose last EXEC has not finished: the pack kernels,
    // which overwrite them, wait for it on this stream (the copy into the staging area need not).
    for (int32_t pg : m->pages) {
        hipEvent_t guard = c->page_guard[pg];
        if (!guard) continue;
        const hipError_t q = hipEventQuery(guard);
        if (q == hipErrorNotReady && (e = hipStreamWaitEvent(st, guard, 0)) != hipSuccess) return bail(e, "hipStreamWaitEvent");
        if (q != hipSuccess && q != hipErrorNotReady) return bail(q, "hipEventQuery");
        for (int32_t pg2 : m->pages)
            if (c->page_guard[pg2] == guard) c->page_guard[pg2] = nullptr;   // waited for (or over) once for all of them
    }
    auto at = [&](size_t off) { return c->pool + (size_t)m->pages[off / c->page_bytes] * c->page_bytes + off % c->page_bytes; };
    for (const WeightSlot &ws : m->m.wslots) {
        const bool is_conv = m->m.ops[ws.op_index].op == CW_OP_CONV;
        if (ws.depthwise)
            e = launch_pack_depthwise(c->staging + ws.blob_w_off, at(ws.packed_w_off), ws.cout, ws.kh, ws.kw, st);
        else
            e = launch_pack_weights(c->staging + ws.blob_w_off, at(ws.packed_w_off), ws.cout, ws.cin, ws.kh, ws.kw, ws.khp,
                                    ws.kwp, ws.cinp, is_conv, st);
        if (e != hipSuccess) return bail(e, "pack_weights");
        if (ws.wino_bytes) {
            e = launch_pack_winograd(m->m.dtype, c->staging + ws.blob_w_off, at(ws.wino_w_off), ws.cout, ws.cin, st);
            if (e != hipSuccess) return bail(e, "pack_winograd");
        }
        e = launch_copy_f32(reinterpret_cast<const float *>(c->staging + ws.blob_b_off),
                            reinterpret_cast<float *>(at(ws.packed_b_off)), ws.cout, st);
        if (e != hipSuccess) return bail(e, "copy bias");
    }
    // resident programs: every member's arguments with the weights' addresses of this placement;
    // activations stay workspace offsets (res + 1, so that 0 means none)
    m->res_programs.clear();
    for (const Plan &p : m->m.plans)
        for (const Launch &l : p.launches) {
            if (l.kind != K_RESIDENT) continue;
            std::vector<ResLayer> prog(l.members.size());
            for (size_t k = 0; k < l.members.size(); ++k) {
                const Launch &ml = l.members[k];
                ResLayer &r = prog[k];
                r = ResLayer{};
                r.a = ml.conv;
                r.a.x = reinterpret_cast<const void *>(ml.x.offset);
                r.a.y = reinterpret_cast<void *>(ml.y.offset);
                r.a.res = ml.res.space == SP_WORKSPACE ? reinterpret_cast<const void *>(ml.res.offset + 1) : nullptr;
                r.a.w = at(ml.w.offset);
                r.a.bias = reinterpret_cast<const float *>(at(ml.bias.offset));
                r.a.partial = nullptr; r.a.counters = nullptr;
                r.ps_x = ml.res_ps_x; r.ps_y = ml.res_ps_y; r.ps_res = ml.res_ps_res;
                r.variant = ml.res_variant; r.tiles = ml.res_tiles;
                r.dep[0] = ml.res_dep[0]; r.dep[1] = ml.res_dep[1];
                r.flag_base = ml.res_flag_base;
                if (ml.x.space != SP_WORKSPACE || ml.y.space != SP_WORKSPACE || !resident_layer_ok(r, c->cfg.workspace_bytes) ||
                    r.dep[0] >= (int)k || r.dep[1] >= (int)k || r.flag_base + r.tiles > l.res_flags_per_part)
                    return bail(hipErrorInvalidValue, "resident program does not fit the kernel's assumptions");
            }
            m->res_programs.push_back(std::move(prog));
            const std::vector<ResLayer> &keep = m->res_programs.back();
            if ((e = hipMemcpyAsync(at(l.w.offset), keep.data(), keep.size() * sizeof(ResLayer), hipMemcpyHostToDevice, st)) != hipSuccess)
                return bail(e, "hipMemcpyAsync of a resident program");
        }
    if ((e = hipEventRecord(c->staging_free, st)) != hipSuccess) return bail(e, "hipEventRecord");
    c->staging_used = true;
    if ((e = hipEventRecord(m->load_done, st)) != hipSuccess) return bail(e, "hipEventRecord");
    m->loaded = true;
    // What is left is host work: the graphs of the plans that have none for this placement.
    cw_load_pending *pd = new cw_load_pending;
    pd->model_id = model_id;
    pd->pages = m->pages;
    pd->want.assign(m->m.plans.size(), 0);
    m->active_set = -1;
    for (size_t k = 0; k < m->graph_sets.size(); ++k)
        if (m->graph_sets[k].pages == m->pages) { m->active_set = (int)k; m->graph_sets[k].last_used = ++c->load_counter; }
    if (c->use_graphs)
        for (size_t pi = 0; pi < m->m.plans.size(); ++pi)
            pd->want[pi] = !(m->active_set >= 0 && m->graph_sets[m->active_set].plans[pi].exec);
    *pending = pd;
    return CW_OK;
}

int32_t cw_load_weights_record(cw_ctx *c, cw_load_pending *pd) {
    if (!c || !pd) return CW_ERR_INVALID;
    const ModelRt *m = get_model(c, pd->model_id);
    if (!m) return CW_ERR_INVALID;
    DeviceGuard g(c->device);
    pd->status = record_graphs(c, m, pd->pages, pd->want, &pd->graphs, &pd->err);
    return pd->status;
}

int32_t cw_load_weights_end(cw_ctx *c, cw_load_pending *pd) {
    if (!c || !pd) return CW_ERR_INVALID;
    ModelRt *m = get_model(c, pd->model_id);
    if (!m) return set_err(c, CW_ERR_INVALID, "unknown model id");
    if (pd->status != CW_OK) return set_err(c, pd->status, pd->err);  // LOAD stays valid; EXEC issues plain launches
    if (!m->loaded || m->pages != pd->pages) return CW_OK;            // unloaded meanwhile: the graphs are of no use
    bool any = false;
    for (const PlanGraph &g : pd->graphs) any = any || g.exec;
    if (!any) return CW_OK;
    if (m->active_set < 0) {
        if (m->graph_sets.size() >= kMaxGraphSets) {  // the placement used longest ago makes room; `pd` takes its graphs along
            size_t old = 0;
            for (size_t k = 1; k < m->graph_sets.size(); ++k)
                if (m->graph_sets[k].last_used < m->graph_sets[old].last_used) old = k;
            for (PlanGraph &g : m->graph_sets[old].plans)
                if (g.exec) pd->graphs.push_back(g);
            m->graph_sets.erase(m->graph_sets.begin() + old);
        }
        GraphSet gs;
        gs.pages = pd->pages;
        gs.plans.resize(m->m.plans.size());
        gs.last_used = ++c->load_counter;
        m->graph_sets.push_back(std::move(gs));
        m->active_set = (int)m->graph_sets.size() - 1;
    }
    GraphSet &gs = m->graph_sets[m->active_set];
    for (size_t pi = 0; pi < gs.plans.size(); ++pi)
        if (pd->graphs[pi].exec && !gs.plans[pi].exec) { gs.plans[pi] = pd->graphs[pi]; pd->graphs[pi].exec = nullptr; }
    return CW_OK;
}

void cw_load_weights_release(cw_load_pending *pd) {
    if (!pd) return;
    destroy_graphs(pd->graphs);
    delete pd;
}

int32_t cw_load_weights(cw_ctx *c, int32_t model_id, const void *host_blob, size_t bytes, void *stream) {
    cw_load_pending *pd = nullptr;
    int32_t rc = cw_load_weights_begin(c, model_id, host_blob, bytes, stream, &pd);
    if (rc != CW_OK) return rc;
    (void)cw_load_weights_record(c, pd);
    (void)cw_load_weights_end(c, pd);   // a recording that failed leaves the LOAD valid: EXEC then issues plain launches
    cw_load_weights_release(pd);
    return CW_OK;
}

int32_t cw_unload_weights(cw_ctx *c, int32_t model_id) {
    ModelRt *m = get_model(c, model_id);
    if (!m) return set_err(c, CW_ERR_INVALID, "unknown model id");
    if (m->loaded) {
        release_pages(c, m);
        m->loaded = false;
    }
    return CW_OK;
}

int32_t cw_input(cw_ctx *c, int32_t model_id, int32_t batch, const float *host_nchw, int32_t *slot, void *stream) {
    if (!c) return CW_ERR_INVALID;
    if (c->device < 0) return set_err(c, CW_ERR_INVALID, "planning-only context has no device");
    ModelRt *m = get_model(c, model_id);
    if (!m || !host_nchw || !slot) return set_err(c, CW_ERR_INVALID, "unknown model id or null pointer");
    if (!get_plan(m, batch)) return set_err(c, CW_ERR_BAD_BATCH, "no plan for this batch size");
    DeviceGuard g(c->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t idx = -1;
    int32_t rc = acquire_slot(c, m, model_id, batch, st, &idx);
    if (rc != CW_OK) return rc;
    Slot &s = c->slots[idx];
    const size_t in_b = (size_t)batch * m->m.in_c * m->m.in_h * m->m.in_w * 4;
    hipError_t e = hipMemcpyAsync(c->io + s.in_off, host_nchw, in_b, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipEventRecord(s.input_done, st);
    if (e != hipSuccess) {
        free_slot(c, &s);
        return hip_fail(c, e, "input copy");
    }
    *slot = idx;
    return CW_OK;
}

int32_t cw_exec(cw_ctx *c, int32_t model_id, int32_t batch, int32_t slot, void *stream) {
    ModelRt *m; Plan *p; Slot *s;
    int32_t rc = exec_checks(c, model_id, batch, slot, &m, &p, &s);
    if (rc != CW_OK) return rc;
    DeviceGuard g(c->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = exec_gate(c, m, s, st);
    if (rc != CW_OK) return rc;
    CW_HIP(c, hipEventRecord(s->exec_start, st));
    rc = enqueue_plan(c, m, p, s, st);
    if (rc != CW_OK) return rc;
    CW_HIP(c, hipEventRecord(s->exec_end, st));
    s->state = SLOT_EXECUTED;
    c->last_exec_stream = st;
    c->last_exec_end = s->exec_end;
    m->last_exec_end = s->exec_end;
    return CW_OK;
}

int32_t cw_exec_static(cw_ctx *c, int32_t model_id, int32_t batch, const float *dev_input_nchw, float *dev_logits,
                       float *dev_probs, void *stream) {
    if (!c) return CW_ERR_INVALID;
    if (c->device < 0) return set_err(c, CW_ERR_INVALID, "planning-only context has no device");
    ModelRt *m = get_model(c, model_id);
    if (!m) return set_err(c, CW_ERR_INVALID, "unknown model id");
    Plan *p = get_plan(m, batch);
    if (!p) return set_err(c, CW_ERR_BAD_BATCH, "no plan for this batch size");
    if (!m->loaded) return set_err(c, CW_ERR_NOT_LOADED, "weights are not resident");
    if (!dev_input_nchw || !dev_logits || !dev_probs) return set_err(c, CW_ERR_INVALID, "null device buffer");
    if (p->workspace_bytes > kStaticScratchBytes) {
        char buf[160];
        snprintf(buf, sizeof buf, "plan needs %zu bytes of intermediates, the static arena holds %zu", p->workspace_bytes,
                 kStaticScratchBytes);
        return set_err(c, CW_ERR_NO_MEMORY, buf);
    }
    if (!c->static_scratch) return set_err(c, CW_ERR_HIP, "static arena has no address on this device");
    DeviceGuard g(c->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The weights must have landed.  A LOAD that has completed needs no stream operation at all.
    const hipError_t q = hipEventQuery(m->load_done);
    if (q == hipErrorNotReady) CW_HIP(c, hipStreamWaitEvent(st, m->load_done, 0));
    else if (q != hipSuccess) return hip_fail(c, q, "hipEventQuery");
    Bases b;
    b.workspace = c->static_scratch;
    b.pages = m->pages.data();
    b.input = const_cast<char *>(reinterpret_cast<const char *>(dev_input_nchw));
    b.logits = reinterpret_cast<char *>(dev_logits);
    b.probs = reinterpret_cast<char *>(dev_probs);
    // The arena keeps what the last call left: the split-K arrival counters at its start must be
    // zero (a fill kernel, not a memset, so that the call may be recorded into a graph).
    hipError_t e = launch_fill_zero(c->static_scratch, kCounterBytes, st);
    if (e != hipSuccess) return hip_fail(c, e, "clearing the arrival counters");
    for (const Launch &l : p->launches) {
        e = issue(c, m, b, l, st);
        if (e != hipSuccess) return hip_fail(c, e, l.info.name);
    }
    return CW_OK;
}

size_t cw_exec_static_capacity(void) { return kStaticScratchBytes; }

int32_t cw_set_use_graphs(cw_ctx *c, int32_t on) {
    if (!c) return CW_ERR_INVALID;
    c->use_graphs = on != 0;
    return CW_OK;
}

int32_t cw_exec_timed_launches(cw_ctx *c, int32_t model_id, int32_t batch, int32_t slot, int32_t inner, float *launch_us,
                               void *stream) {
    ModelRt *m; Plan *p; Slot *s;
    int32_t rc = exec_checks(c, model_id, batch, slot, &m, &p, &s);
    if (rc != CW_OK) return rc;
    if (!launch_us || inner < 1) return set_err(c, CW_ERR_INVALID, "null output or inner < 1");
    DeviceGuard g(c->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = exec_gate(c, m, s, st);
    if (rc != CW_OK) return rc;
    const size_t n = p->launches.size();
    CW_HIP(c, hipEventRecord(s->exec_start, st));
    for (size_t base = 0; base < n; base += kProfileEvents) {
        const size_t cnt = std::min<size_t>(kProfileEvents, n - base);
        for (size_t i = 0; i < cnt; ++i) {
            CW_HIP(c, hipEventRecord(c->prof_ev[2 * i], st));
            for (int r = 0; r < inner; ++r) {
                hipError_t e = issue(c, m, bases_of(c, m, s), p->launches[base + i], st);
                if (e != hipSuccess) return hip_fail(c, e, p->launches[base + i].info.name);
            }
            CW_HIP(c, hipEventRecord(c->prof_ev[2 * i + 1], st));
        }
        CW_HIP(c, hipStreamSynchronize(st));
        for (size_t i = 0; i < cnt; ++i) {
            float ms = 0.f;
            CW_HIP(c, hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]));
            launch_us[base + i] = ms * 1000.f / (float)inner;
        }
    }
    CW_HIP(c, hipEventRecord(s->exec_end, st));
    CW_HIP(c, hipStreamSynchronize(st));
    s->state = SLOT_EXECUTED;
    c->last_exec_stream = st;
    c->last_exec_end = s->exec_end;
    return CW_OK;
}

int32_t cw_output(cw_ctx *c, int32_t slot, float *host_probs, float *host_logits, void *stream) {
    if (!c) return CW_ERR_INVALID;
    if (c->device < 0) return set_err(c, CW_ERR_INVALID, "planning-only context has no device");
    if (slot < 0 || slot >= kMaxSlots || c->slots[slot].state != SLOT_EXECUTED)
        return set_err(c, CW_ERR_NO_INPUT, "slot holds no result");
    if (!host_probs) return set_err(c, CW_ERR_INVALID, "null output buffer");
    Slot &s = c->slots[slot];
    ModelRt *m = get_model(c, s.model);
    DeviceGuard g(c->device);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t out_b = (size_t)s.batch * m->m.classes * 4;
    CW_HIP(c, hipStreamWaitEvent(st, s.exec_end, 0));
    CW_HIP(c, hipMemcpyAsync(host_probs, c->io + s.probs_off, out_b, hipMemcpyDeviceToHost, st));
    if (host_logits) CW_HIP(c, hipMemcpyAsync(host_logits, c->io + s.logits_off, out_b, hipMemcpyDeviceToHost, st));
    CW_HIP(c, hipEventRecord(s.released, st));
    s.release_pending = true;
    free_slot(c, &s);
    return CW_OK;
}

int32_t cw_release(cw_ctx *c, int32_t slot) {
    if (!c || slot < 0 || slot >= kMaxSlots) return set_err(c, CW_ERR_INVALID, "bad slot");
    Slot &s = c->slots[slot];
    if (s.state == SLOT_FREE) return CW_OK;
    if (c->device >= 0) {
        // Work that reads or writes the slot may still be queued: whoever reuses the memory waits
        // for the last EXEC that touched it.
        DeviceGuard g(c->device);
        if (s.state == SLOT_EXECUTED) {
            CW_HIP(c, hipStreamWaitEvent(c->internal_stream, s.exec_end, 0));
            CW_HIP(c, hipEventRecord(s.released, c->internal_stream));
            s.release_pending = true;
        }
    }
    free_slot(c, &s);
    return CW_OK;
}

int32_t cw_exec_duration_ns(cw_ctx *c, int32_t slot, uint64_t *ns) {
    if (!c || !ns) return CW_ERR_INVALID;
    if (slot < 0 || slot >= kMaxSlots || c->slots[slot].state != SLOT_EXECUTED)
        return set_err(c, CW_ERR_NO_INPUT, "slot holds no result");
    Slot &s = c->slots[slot];
    DeviceGuard g(c->device);
    CW_HIP(c, hipEventSynchronize(s.exec_end));
    float ms = 0.f;
    CW_HIP(c, hipEventElapsedTime(&ms, s.exec_start, s.exec_end));
    *ns = (uint64_t)((double)ms * 1e6 + 0.5);
    if (c->res_error && *reinterpret_cast<volatile unsigned *>(c->res_error) != 0u)
        return set_err(c, CW_ERR_HIP, *c->res_error == 2u ? "a resident launch found a workgroup on an unexpected XCD: results are invalid"
                                                          : "a resident launch gave up waiting for a layer: results are invalid");
    return CW_OK;
}

int32_t cw_profile_measure(cw_ctx *c, int32_t model_id, int32_t batch, int32_t slot, uint32_t repeats, cw_profile *out,
                           float *samples_us) {
    if (!c || !out || repeats == 0) return set_err(c, CW_ERR_INVALID, "null output or zero repeats");
    if (c->device < 0) return set_err(c, CW_ERR_INVALID, "planning-only context has no device");
    ModelRt *m = get_model(c, model_id);
    if (!m) return set_err(c, CW_ERR_INVALID, "unknown model id");
    Plan *p = get_plan(m, batch);
    if (!p) return set_err(c, CW_ERR_BAD_BATCH, "no plan for this batch size");
    if (!m->loaded) return set_err(c, CW_ERR_NOT_LOADED, "weights are not resident");
    DeviceGuard g(c->device);
    hipStream_t st = c->internal_stream;
    if (c->last_exec_end) CW_HIP(c, hipEventSynchronize(c->last_exec_end));  // one EXEC at a time
    // The input the EXECs run over: the caller's slot (EXEC time depends a little on the values,
    // through power and clocks), or a zero-filled one of the library's own.
    const bool own_slot = slot < 0;
    hipError_t e = hipSuccess;
    int32_t rc = CW_OK;
    if (own_slot) {
        rc = acquire_slot(c, m, model_id, batch, st, &slot);
        if (rc != CW_OK) return rc;
        const size_t in_b = ((size_t)batch * m->m.in_c * m->m.in_h * m->m.in_w * 4 + 255) / 256 * 256;
        e = launch_fill_zero(c->io + c->slots[slot].in_off, in_b, st);
        if (e == hipSuccess) e = hipEventRecord(c->slots[slot].input_done, st);
    } else {
        if (slot >= kMaxSlots || c->slots[slot].state == SLOT_FREE) return set_err(c, CW_ERR_NO_INPUT, "slot holds no input");
        if (c->slots[slot].model != model_id) return set_err(c, CW_ERR_NO_INPUT, "slot holds an input for another model");
        if (c->slots[slot].batch != batch) return set_err(c, CW_ERR_BAD_BATCH, "slot holds an input of another batch size");
        e = hipStreamWaitEvent(st, c->slots[slot].input_done, 0);
    }
    Slot &s = c->slots[slot];
    if (e == hipSuccess) e = hipStreamWaitEvent(st, m->load_done, 0);
    if (e != hipSuccess) {
        if (own_slot) free_slot(c, &s);
        return hip_fail(c, e, "profile setup");
    }
    std::vector<float> samples;
    samples.reserve(repeats);
    for (uint32_t done = 0; done < repeats && rc == CW_OK;) {
        const uint32_t cnt = std::min<uint32_t>(kProfileEvents, repeats - done);
        // One untimed EXEC leads every burst: without it the first start event of a burst fires on
        // an idle GPU while the host is still submitting the work it is meant to time.
        rc = enqueue_plan(c, m, p, &s, st);
        for (uint32_t i = 0; i < cnt && rc == CW_OK; ++i) {
            if ((e = hipEventRecord(c->prof_ev[2 * i], st)) != hipSuccess) { rc = hip_fail(c, e, "hipEventRecord"); break; }
            rc = enqueue_plan(c, m, p, &s, st);
            if (rc == CW_OK && (e = hipEventRecord(c->prof_ev[2 * i + 1], st)) != hipSuccess) rc = hip_fail(c, e, "hipEventRecord");
        }
        if ((e = hipStreamSynchronize(st)) != hipSuccess && rc == CW_OK) rc = hip_fail(c, e, "hipStreamSynchronize");
        for (uint32_t i = 0; i < cnt && rc == CW_OK; ++i) {
            float ms = 0.f;
            if ((e = hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1])) != hipSuccess) { rc = hip_fail(c, e, "hipEventElapsedTime"); break; }
            samples.push_back(ms * 1000.f);
        }
        done += cnt;
    }
    if (own_slot) free_slot(c, &s);
    if (rc != CW_OK) return rc;
    percentile_profile(samples, &p->profile);
    *out = p->profile;
    if (samples_us) std::copy(samples.begin(), samples.end(), samples_us);
    return CW_OK;
}

int32_t cw_profile_get(cw_ctx *c, int32_t model_id, int32_t batch, cw_profile *out) {
    ModelRt *m = get_model(c, model_id);
    if (!m || !out) return set_err(c, CW_ERR_INVALID, "unknown model id");
    Plan *p = get_plan(m, batch);
    if (!p) return set_err(c, CW_ERR_BAD_BATCH, "no plan for this batch size");
    *out = p->profile;
    return CW_OK;
}

int32_t cw_plan_num_launches(cw_ctx *c, int32_t model_id, int32_t batch) {
    ModelRt *m = get_model(c, model_id);
    if (!m) return set_err(c, CW_ERR_INVALID, "unknown model id");
    Plan *p = get_plan(m, batch);
    if (!p) return set_err(c, CW_ERR_BAD_BATCH, "no plan for this batch size");
    return (int32_t)p->launches.size();
}

int32_t cw_plan_launch_info(cw_ctx *c, int32_t model_id, int32_t batch, int32_t index, cw_launch_info *out) {
    ModelRt *m = get_model(c, model_id);
    if (!m || !out) return set_err(c, CW_ERR_INVALID, "unknown model id");
    Plan *p = get_plan(m, batch);
    if (!p) return set_err(c, CW_ERR_BAD_BATCH, "no plan for this batch size");
    if (index < 0 || index >= (int32_t)p->launches.size()) return set_err(c, CW_ERR_INVALID, "launch index out of range");
    *out = p->launches[index].info;
    return CW_OK;
}

int32_t cw_debug_read_op(cw_ctx *c, int32_t model_id, int32_t batch, int32_t op_index, float *host_out, size_t cap) {
    if (!c || !host_out) return CW_ERR_INVALID;
    if (c->device < 0) return set_err(c, CW_ERR_INVALID, "planning-only context has no device");
    ModelRt *m = get_model(c, model_id);
    if (!m) return set_err(c, CW_ERR_INVALID, "unknown model id");
    Plan *p = get_plan(m, batch);
    if (!p) return set_err(c, CW_ERR_BAD_BATCH, "no plan for this batch size");
    if (!m->m.keep_all) return set_err(c, CW_ERR_UNSUPPORTED, "model was not defined with debug retention");
    if (op_index < 0 || op_index >= (int32_t)m->m.ops.size()) return set_err(c, CW_ERR_INVALID, "bad op index");
    const Ref &r = p->op_out[op_index];
    if (r.space == SP_NONE) return set_err(c, CW_ERR_UNSUPPORTED, "op is computed inside a fused launch; its output is never stored");
    if (r.space != SP_WORKSPACE) return set_err(c, CW_ERR_UNSUPPORTED, "op output lives in the IO slot; use cw_output");
    const OpShape &sh = m->m.shapes[op_index];
    const size_t count = (size_t)batch * sh.c * sh.h * sh.w;
    if (cap < count) return set_err(c, CW_ERR_INVALID, "host buffer too small");
    DeviceGuard g(c->device);
    CW_HIP(c, hipDeviceSynchronize());
    if (m->m.ops[op_index].op == CW_OP_GAVGPOOL) {  // already fp32 [B][C]
        CW_HIP(c, hipMemcpy(host_out, c->workspace + r.offset, count * 4, hipMemcpyDeviceToHost));
        return CW_OK;
    }
    // The conversion needs count*4 bytes of scratch: the LOAD staging area is idle after the sync.
    if (count * 4 > c->cfg.load_staging_bytes) return set_err(c, CW_ERR_NO_MEMORY, "staging area too small for read-back");
    hipError_t e = launch_nhwc_to_nchw_f32(m->m.dtype, c->workspace + r.offset, reinterpret_cast<float *>(c->staging), batch,
                                           sh.c, sh.h, sh.w, p->op_ld[op_index], c->internal_stream);
    if (e != hipSuccess) return hip_fail(c, e, "nhwc_to_nchw");
    CW_HIP(c, hipStreamSynchronize(c->internal_stream));
    CW_HIP(c, hipMemcpy(host_out, c->staging, count * 4, hipMemcpyDeviceToHost));
    return CW_OK;
}

}  // extern "C"
