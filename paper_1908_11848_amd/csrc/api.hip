// C ABI of libdssp: context, the server's decision logic (Alg. 1 server part, Alg. 2) on the
// host, and the stream / event ordering between the applies and the K workers' streams.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <map>
#include <tuple>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "../../include/dssp.h"
#include "../../include/dssp_kernels.h"
#include "model.hpp"

struct dssp_ctx {
    int K = 0, s_L = 0, r_max = 0;
    float lr = 0.f, scale = 0.f;
    bool host_only = false;
    float* params = nullptr;
    int64_t n_params = 0;

    // Alg. 1 preamble and Alg. 2 table A
    std::vector<int64_t> t;                       // pushes received per worker
    std::vector<int32_t> r;                       // extra-iteration credit per worker
    std::vector<std::array<int64_t, 2>> A;        // [latest, second latest] push timestamp
    std::vector<uint8_t> blocked;                 // waiting for a postponed OK
    std::vector<uint8_t> has_ok;                  // may pull and run one iteration
    uint64_t version = 0;                         // number of applies

    // device side
    hipStream_t server_stream = nullptr;
    std::vector<hipStream_t> wstream;
    std::vector<uint8_t> own_wstream;
    hipEvent_t ev_apply = nullptr;                // last apply finished
    std::vector<hipEvent_t> ev_grad;              // worker's gradient is complete
    std::vector<hipEvent_t> ev_pull;              // worker's snapshot copy finished reading w
    std::vector<uint8_t> pull_pending;            // a pull was enqueued since the last apply
    uint64_t* stamps_dev = nullptr;               // [0] global stamp, [1+p] stamp of p's snapshot

    // wall-clock mode (dssp_worker_step_timed / dssp_step_done); set up on first use
    uint64_t* ticks_host = nullptr;               // pinned: per worker [start, gradient finished, stream released, unused]
    uint64_t* ticks_dev = nullptr;                // the same memory as the device addresses it
    std::vector<hipEvent_t> ev_done;              // worker's timed step (and its hold) has left the stream
    std::vector<uint8_t> timed_pending;
    int wall_khz = 0;
    uint64_t origin_tick = 0;                     // tick that counts as time 0

    int model_id = DSSP_MODEL_NONE;
    dssp_model::Plan* plan = nullptr;

    // A worker step is a fixed chain of several hundred kernels whose arguments depend only on the
    // five buffers it is called with.  The first call with a set of buffers runs eagerly, the second
    // is captured into a HIP graph, later ones replay the graph (one submission instead of hundreds).
    struct StepGraph { int calls = 0; hipGraph_t graph = nullptr; hipGraphExec_t exec = nullptr; };
    typedef std::tuple<int, const void*, const void*, const void*, const void*, const void*> StepKey;
    std::map<StepKey, StepGraph> step_graphs;
    bool use_graphs = true;

    std::string err;
};

namespace {

int fail(dssp_ctx* c, int code, const std::string& msg) {
    if (c) c->err = msg;
    return code;
}

#define HIP_TRY(c, expr)                                                                      \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail((c), DSSP_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_));   \
    } while (0)

// Slowest worker: fewest pushes; among those the one whose latest push is oldest; then lowest index.
int find_slowest(const dssp_ctx* c) {
    int s = 0;
    for (int i = 1; i < c->K; ++i) {
        if (c->t[i] != c->t[s]) {
            if (c->t[i] < c->t[s]) s = i;
        } else if (c->A[i][0] < c->A[s][0]) {
            s = i;
        }
    }
    return s;
}

// floor(a / b) for b > 0
__int128 floor_div(__int128 a, __int128 b) {
    __int128 q = a / b;
    if ((a % b != 0) && (a < 0)) --q;
    return q;
}

// Alg. 2 from step 3 on (table A was shifted when the push arrived).  Extrapolates r_max+1 push times of p (from its
// current push) and of the slowest worker (from one interval after its latest push) and returns the index on p's
// timeline that comes closest to any push of the slowest worker; of equally close ones the smallest.  Both timelines
// are arithmetic progressions, so for each of p's r_max+1 times the closest time of the slowest worker is found by
// one division (its two neighbours in the progression, clamped to the ends) instead of a scan: O(r_max) per call
// where the double loop of the algorithm as printed is O(r_max^2), with the same result (tested against that loop).
int synchronization_controller(const dssp_ctx* c, int p) {
    const int slow = find_slowest(c);
    const __int128 ip = c->A[p][0] - c->A[p][1];
    const __int128 is = c->A[slow][0] - c->A[slow][1];
    const __int128 s0 = (__int128)c->A[slow][0] + is;          // Sim_slowest[k] = s0 + k * is, k = 0 .. r_max
    const __int128 step = is < 0 ? -is : is;
    const __int128 lo = is < 0 ? s0 + (__int128)c->r_max * is : s0;      // the same set of times, ascending: lo + j * step
    int r_star = 0;
    bool have = false;
    __int128 best = 0;
    for (int rr = 0; rr <= c->r_max; ++rr) {
        const __int128 sp = (__int128)c->A[p][0] + (__int128)rr * ip;
        __int128 d;
        if (step == 0) {
            d = sp > lo ? sp - lo : lo - sp;
        } else {
            __int128 j = floor_div(sp - lo, step);
            if (j < 0) j = 0;
            if (j > c->r_max) j = c->r_max;
            const __int128 a = lo + j * step;
            d = sp > a ? sp - a : a - sp;
            if (j < c->r_max) {
                const __int128 b = a + step;
                const __int128 db = sp > b ? sp - b : b - sp;
                if (db < d) d = db;
            }
        }
        if (!have || d < best) { have = true; best = d; r_star = rr; }
    }
    return r_star;
}

void drop_step_graphs(dssp_ctx* c) {
    for (auto& kv : c->step_graphs) {
        if (kv.second.exec) (void)hipGraphExecDestroy(kv.second.exec);
        if (kv.second.graph) (void)hipGraphDestroy(kv.second.graph);
    }
    c->step_graphs.clear();
}

int check_worker(dssp_ctx* c, int worker) {
    if (!c) return DSSP_EINVAL;
    if (worker < 0 || worker >= c->K) return fail(c, DSSP_EINVAL, "worker index out of range");
    return DSSP_OK;
}

}  // namespace

extern "C" int dssp_create(dssp_ctx** out, float* params_dev, int64_t n_params, int K, int s_L, int r_max, float lr) {
    if (!out) return DSSP_EINVAL;
    *out = nullptr;
    if (K < 1 || K > 4096 || s_L < 0 || r_max < 0 || r_max > 1 << 20 || n_params < 0) return DSSP_EINVAL;
    if ((params_dev == nullptr) != (n_params == 0)) return DSSP_EINVAL;
    dssp_ctx* c = new dssp_ctx();
    c->K = K; c->s_L = s_L; c->r_max = r_max; c->lr = lr;
    c->scale = lr / (float)K;
    c->host_only = params_dev == nullptr;
    c->params = params_dev; c->n_params = n_params;
    if (const char* e = std::getenv("DSSP_NO_GRAPH")) c->use_graphs = !(e[0] && e[0] != '0');
    c->t.assign(K, 0); c->r.assign(K, 0); c->A.assign(K, {0, 0});
    c->blocked.assign(K, 0); c->has_ok.assign(K, 1);
    c->wstream.assign(K, nullptr); c->own_wstream.assign(K, 0);
    c->ev_grad.assign(K, nullptr); c->ev_pull.assign(K, nullptr); c->pull_pending.assign(K, 0);
    *out = c;
    if (c->host_only) return DSSP_OK;
    hipError_t e = hipMalloc((void**)&c->stamps_dev, sizeof(uint64_t) * (K + 1));
    if (e == hipSuccess) e = hipMemset(c->stamps_dev, 0, sizeof(uint64_t) * (K + 1));
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_apply, hipEventDisableTiming);
    for (int p = 0; p < K && e == hipSuccess; ++p) {
        e = hipEventCreateWithFlags(&c->ev_grad[p], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_pull[p], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        std::fprintf(stderr, "dssp_create: %s\n", hipGetErrorString(e));
        dssp_destroy(c);
        *out = nullptr;
        return DSSP_EHIP;
    }
    return DSSP_OK;
}

namespace {
// Worker streams the caller did not set are created on first use.
int ensure_stream(dssp_ctx* c, int worker) {
    if (c->host_only) return DSSP_OK;
    hipStream_t& s = c->wstream[worker];
    if (s) return DSSP_OK;
    HIP_TRY(c, hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
    c->own_wstream[worker] = 1;
    return DSSP_OK;
}
}  // namespace

extern "C" int dssp_set_stream(dssp_ctx* c, int worker, void* hip_stream) {
    if (!c) return DSSP_EINVAL;
    if (worker < -1 || worker >= c->K) return fail(c, DSSP_EINVAL, "worker index out of range");
    if (c->host_only) return DSSP_OK;
    if (worker < 0) { c->server_stream = (hipStream_t)hip_stream; return DSSP_OK; }
    hipStream_t& s = c->wstream[worker];
    if (c->own_wstream[worker] && s) { HIP_TRY(c, hipStreamSynchronize(s)); HIP_TRY(c, hipStreamDestroy(s)); }
    s = (hipStream_t)hip_stream;
    c->own_wstream[worker] = 0;
    return DSSP_OK;
}

extern "C" int dssp_set_model(dssp_ctx* c, int model_id, int batch, int n_classes, void* workspace_dev, size_t workspace_bytes) {
    if (!c) return DSSP_EINVAL;
    if (c->host_only) return fail(c, DSSP_ESTATE, "host-only context has no model");
    if (c->plan) {
        if (int rc = dssp_synchronize(c)) return rc;
        drop_step_graphs(c);
        dssp_model::destroy(c->plan); c->plan = nullptr; c->model_id = DSSP_MODEL_NONE;
    }
    if (model_id == DSSP_MODEL_NONE) return DSSP_OK;
    const int64_t np = dssp_model_param_count(model_id, n_classes);
    if (np < 0 || batch < 1 || n_classes < 2) return fail(c, DSSP_EINVAL, "unknown model, batch < 1 or n_classes < 2");
    if (np != c->n_params) return fail(c, DSSP_EINVAL, "n_params of the context does not match the model");
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255))
        return fail(c, DSSP_EINVAL, "workspace must be non-null and 256-byte aligned");
    if (workspace_bytes < dssp_workspace_bytes(model_id, batch, n_classes, c->K))
        return fail(c, DSSP_ENOMEM, "workspace smaller than dssp_workspace_bytes()");
    std::string err;
    c->plan = dssp_model::create(model_id, batch, n_classes, c->K, workspace_dev, err);
    if (!c->plan) return fail(c, DSSP_EINVAL, err);
    c->model_id = model_id;
    return DSSP_OK;
}

extern "C" int dssp_pull(dssp_ctx* c, int worker, float* dst_dev, uint64_t* version_out) {
    if (int rc = check_worker(c, worker)) return rc;
    if (!c->has_ok[worker]) return fail(c, DSSP_ESTATE, "pull by a worker that holds no OK");
    if (version_out) *version_out = c->version;
    if (c->host_only) return DSSP_OK;
    if (!dst_dev) return fail(c, DSSP_EINVAL, "dst_dev is null");
    if (int rc = ensure_stream(c, worker)) return rc;
    hipStream_t s = c->wstream[worker];
    if (c->version > 0) HIP_TRY(c, hipStreamWaitEvent(s, c->ev_apply, 0));
    if (int rc = dsspk_pull(s, dst_dev, c->params, c->n_params, c->stamps_dev + 1 + worker, c->stamps_dev))
        return fail(c, DSSP_EHIP, "pull kernel launch failed (rc " + std::to_string(rc) + ")");
    HIP_TRY(c, hipEventRecord(c->ev_pull[worker], s));
    c->pull_pending[worker] = 1;
    return DSSP_OK;
}

extern "C" int dssp_worker_step(dssp_ctx* c, int worker, const float* x_dev, const int32_t* y_dev,
                                const float* w_local_dev, float* grad_dev, float* loss_dev) {
    if (int rc = check_worker(c, worker)) return rc;
    if (c->host_only || !c->plan) return fail(c, DSSP_ESTATE, "worker_step before set_model");
    if (!x_dev || !y_dev || !w_local_dev || !grad_dev) return fail(c, DSSP_EINVAL, "null device pointer");
    if (int rc = ensure_stream(c, worker)) return rc;
    std::string err;
    hipStream_t s = c->wstream[worker];
    dssp_ctx::StepGraph* sg = nullptr;
    if (c->use_graphs) {
        sg = &c->step_graphs[dssp_ctx::StepKey(worker, x_dev, y_dev, w_local_dev, grad_dev, loss_dev)];
        if (sg->exec) {
            HIP_TRY(c, hipGraphLaunch(sg->exec, s));
            return DSSP_OK;
        }
    }
    const bool capture = sg && sg->calls >= 1;
    if (capture) HIP_TRY(c, hipStreamBeginCapture(s, hipStreamCaptureModeRelaxed));
    const int rc = dssp_model::step(c->plan, worker, s, x_dev, y_dev, w_local_dev, grad_dev, loss_dev, err);
    if (capture) {
        hipGraph_t graph = nullptr;
        const hipError_t e = hipStreamEndCapture(s, &graph);
        if (rc || e != hipSuccess) {
            if (graph) (void)hipGraphDestroy(graph);
            return fail(c, DSSP_EHIP, "worker_step (capture): " + err + " rc " + std::to_string(rc) + " " + hipGetErrorString(e));
        }
        const hipError_t ei = hipGraphInstantiate(&sg->exec, graph, nullptr, nullptr, 0);
        if (ei != hipSuccess) {             // the next call with these buffers captures again
            (void)hipGraphDestroy(graph);
            sg->exec = nullptr;
            return fail(c, DSSP_EHIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(ei));
        }
        sg->graph = graph;
        HIP_TRY(c, hipGraphLaunch(sg->exec, s));
        return DSSP_OK;
    }
    if (rc) return fail(c, DSSP_EHIP, "worker_step: " + err + " (rc " + std::to_string(rc) + ")");
    if (sg) sg->calls += 1;
    return DSSP_OK;
}

namespace {

// The integers the server keeps (Alg. 1 preamble, table A of Alg. 2) plus the bookkeeping of pending snapshots: saved
// before a push is decided and put back if any device call of that push fails, so that a failed push leaves the
// context as it was (the clocks never say "applied" for a gradient that was not).
struct HostState {
    std::vector<int64_t> t;
    std::vector<int32_t> r;
    std::vector<std::array<int64_t, 2>> A;
    std::vector<uint8_t> blocked, has_ok, pull_pending;
    uint64_t version;
};

HostState save_state(const dssp_ctx* c) { return HostState{c->t, c->r, c->A, c->blocked, c->has_ok, c->pull_pending, c->version}; }

void restore_state(dssp_ctx* c, const HostState& h) {
    c->t = h.t; c->r = h.r; c->A = h.A; c->blocked = h.blocked; c->has_ok = h.has_ok; c->pull_pending = h.pull_pending;
    c->version = h.version;
}

struct Decision {
    bool ok = false;
    int r_star = -1, grant = -1;
    int n_released = 0;             // written to released[0 .. n_released)
};

// Alg. 1, server part, for the push of worker p at time t_push: everything but the weight update itself, which the
// caller enqueues.  Pure integer work on the host.
Decision decide(dssp_ctx* c, int p, int64_t t_push, int* released) {
    Decision d;
    // Alg. 2 steps 1-2, done for every push so that A really holds the two latest pushes of all workers
    c->A[p][1] = c->A[p][0];
    c->A[p][0] = t_push;
    c->t[p] += 1;            // Alg. 1 server step 1
    c->version += 1;         // Alg. 1 server step 2 (the apply the caller enqueues)
    if (c->r[p] > 0) {       // steps 3-5: spend one unit of credit
        c->r[p] -= 1;
        d.ok = true;
    } else {
        const int64_t t_min = *std::min_element(c->t.begin(), c->t.end());
        const int64_t t_max = *std::max_element(c->t.begin(), c->t.end());
        const int64_t gap = c->t[p] - t_min;
        if (gap <= c->s_L) {
            d.ok = true;     // steps 8-9
        } else if (c->t[p] == t_max) {
            d.r_star = synchronization_controller(c, p);                      // step 12
            const int64_t room = (int64_t)c->s_L + c->r_max - gap + 1;        // keeps the gap <= s_L + r_max
            d.grant = (int)std::min<int64_t>(d.r_star, room);
            if (d.grant >= 1) { c->r[p] = d.grant - 1; d.ok = true; }         // this OK is the first extra iteration
        }                    // else step 16: wait for the slowest worker
    }
    c->has_ok[p] = d.ok ? 1 : 0;
    c->blocked[p] = d.ok ? 0 : 1;
    const int64_t t_min = *std::min_element(c->t.begin(), c->t.end());
    for (int q = 0; q < c->K; ++q)
        if (q != p && c->blocked[q] && c->t[q] - t_min <= c->s_L) {
            c->blocked[q] = 0;
            c->has_ok[q] = 1;
            released[d.n_released++] = q;
        }
    return d;
}

// Stream `as` waits for the apply before it and for every snapshot copy still reading w.
int wait_for_w(dssp_ctx* c, hipStream_t as, uint64_t applies_before) {
    if (applies_before > 0) HIP_TRY(c, hipStreamWaitEvent(as, c->ev_apply, 0));
    for (int q = 0; q < c->K; ++q)
        if (c->pull_pending[q]) {
            if (c->wstream[q] != as) HIP_TRY(c, hipStreamWaitEvent(as, c->ev_pull[q], 0));
            c->pull_pending[q] = 0;
        }
    return DSSP_OK;
}

// Device half of one push.  The apply runs behind the worker's gradient, behind the apply before it and behind every
// snapshot still reading w.  Without a server stream it goes onto the pusher's own stream, right behind the gradient:
// a separate stream shares a hardware queue with some worker's stream, and the small apply then waits for that
// worker's whole iteration.
int enqueue_apply(dssp_ctx* c, int p, const float* grad_dev, float* pull_dst_dev, bool fused, uint64_t applies_before) {
    const bool own = c->server_stream == nullptr;
    hipStream_t as = own ? c->wstream[p] : c->server_stream;
    if (!own) {
        HIP_TRY(c, hipEventRecord(c->ev_grad[p], c->wstream[p]));
        HIP_TRY(c, hipStreamWaitEvent(as, c->ev_grad[p], 0));
    }
    if (int rc = wait_for_w(c, as, applies_before)) return rc;
    int rc;
    if (fused)      // the worker's stream gets at the snapshot through ev_apply, like at any other pull
        rc = dsspk_apply_pull(as, c->params, grad_dev, pull_dst_dev, c->n_params, c->scale, c->stamps_dev,
                              c->stamps_dev + 1 + p, c->version);
    else
        rc = dsspk_apply(as, c->params, grad_dev, c->n_params, c->scale, c->stamps_dev, c->version);
    if (rc) return fail(c, DSSP_EHIP, "apply kernel launch failed (rc " + std::to_string(rc) + ")");
    HIP_TRY(c, hipEventRecord(c->ev_apply, as));
    if (fused && !own) HIP_TRY(c, hipStreamWaitEvent(c->wstream[p], c->ev_apply, 0));
    return DSSP_OK;
}

// Alg. 1 server part for one push.  The decision (steps 3-16 and Alg. 2) is integer work on the host and does not
// depend on the apply, so it is taken first; the device work enqueued afterwards is the apply alone, or - if the
// pusher may go on at once and handed over where its next snapshot goes - apply and pull in one kernel.
int push_impl(dssp_ctx* c, int worker, const float* grad_dev, int64_t t_push, float* pull_dst_dev, int* ok_out,
              int* released_out, int* n_released_out, int* rstar_out, int* grant_out, int* pulled_out,
              uint64_t* version_out) {
    if (int rc = check_worker(c, worker)) return rc;
    if (!ok_out || !released_out || !n_released_out) return fail(c, DSSP_EINVAL, "null output pointer");
    if (c->blocked[worker] || !c->has_ok[worker])
        return fail(c, DSSP_ESTATE, "push by a worker that is waiting for OK");
    const int p = worker;
    if (!c->host_only) {
        if (!grad_dev) return fail(c, DSSP_EINVAL, "grad_dev is null");
        if (int rc = ensure_stream(c, p)) return rc;
    }
    const HostState before = save_state(c);
    const Decision d = decide(c, p, t_push, released_out);
    const bool fused = d.ok && pull_dst_dev != nullptr;
    if (!c->host_only)
        if (int rc = enqueue_apply(c, p, grad_dev, pull_dst_dev, fused, before.version)) {
            restore_state(c, before);       // nothing of this push counts: the caller may repeat it or give up
            return rc;
        }
    *ok_out = d.ok ? 1 : 0;
    *n_released_out = d.n_released;
    if (rstar_out) *rstar_out = d.r_star;
    if (grant_out) *grant_out = d.grant;
    if (pulled_out) *pulled_out = fused ? 1 : 0;
    if (version_out) *version_out = c->version;
    return DSSP_OK;
}

}  // namespace

extern "C" int dssp_push(dssp_ctx* c, int worker, const float* grad_dev, int64_t t_push, int* ok_out,
                         int* released_out, int* n_released_out, int* rstar_out, int* grant_out) {
    return push_impl(c, worker, grad_dev, t_push, nullptr, ok_out, released_out, n_released_out, rstar_out, grant_out, nullptr,
                     nullptr);
}

extern "C" int dssp_push_pull(dssp_ctx* c, int worker, const float* grad_dev, int64_t t_push, float* pull_dst_dev, int* ok_out,
                              int* released_out, int* n_released_out, int* rstar_out, int* grant_out, int* pulled_out,
                              uint64_t* version_out) {
    if (c && !c->host_only && !pull_dst_dev) return fail(c, DSSP_EINVAL, "pull_dst_dev is null");
    if (!pulled_out) return c ? fail(c, DSSP_EINVAL, "null output pointer") : DSSP_EINVAL;
    static float host_only_dst;           // a host-only context takes the same decisions; the pointer is never used
    return push_impl(c, worker, grad_dev, t_push, (c && c->host_only) ? &host_only_dst : pull_dst_dev, ok_out, released_out,
                     n_released_out, rstar_out, grant_out, pulled_out, version_out);
}

// m pushes with one timestamp: decided one by one in ascending worker order (each decision sees the clocks the pushes
// before it left), applied by one kernel that also hands every worker that may go on after push j the weights as they
// are after push j.
extern "C" int dssp_push_many(dssp_ctx* c, int m, const int* workers, const float* const* grads_dev, int64_t t_push,
                              float* const* pull_dst_dev, int* ok_out, int* rstar_out, int* grant_out, int* n_released_out,
                              int* released_out, uint64_t* pulled_version_out) {
    if (!c) return DSSP_EINVAL;
    if (m < 1 || m > DSSPK_APPLY_MANY_MAX) return fail(c, DSSP_EINVAL, "m must be in [1, " + std::to_string(DSSPK_APPLY_MANY_MAX) + "]");
    if (!workers || !ok_out || !n_released_out || !released_out || !pulled_version_out)
        return fail(c, DSSP_EINVAL, "null pointer");
    if (!c->host_only && (!grads_dev || !pull_dst_dev)) return fail(c, DSSP_EINVAL, "null pointer");
    for (int j = 0; j < m; ++j) {
        if (int rc = check_worker(c, workers[j])) return rc;
        if (j > 0 && workers[j] <= workers[j - 1]) return fail(c, DSSP_EINVAL, "workers must be distinct and ascending");
        if (c->blocked[workers[j]] || !c->has_ok[workers[j]])
            return fail(c, DSSP_ESTATE, "push by a worker that is waiting for OK");
        if (!c->host_only) {
            if (!grads_dev[j]) return fail(c, DSSP_EINVAL, "grad_dev is null");
            if (int rc = ensure_stream(c, workers[j])) return rc;
        }
    }
    const HostState before = save_state(c);
    // snapshots in the order they are taken: after push j its pusher (if it may go on), then the workers it releases
    int snap_worker[DSSPK_APPLY_MANY_MAX_DST], snap_after[DSSPK_APPLY_MANY_MAX_DST], n_snap = 0, n_rel = 0;
    for (int q = 0; q < c->K; ++q) pulled_version_out[q] = 0;
    for (int j = 0; j < m; ++j) {
        const Decision d = decide(c, workers[j], t_push, released_out + n_rel);
        ok_out[j] = d.ok ? 1 : 0;
        if (rstar_out) rstar_out[j] = d.r_star;
        if (grant_out) grant_out[j] = d.grant;
        n_released_out[j] = d.n_released;
        const int first = n_snap;
        if (n_snap + (d.ok ? 1 : 0) + d.n_released > DSSPK_APPLY_MANY_MAX_DST) {
            restore_state(c, before);
            return fail(c, DSSP_EINVAL, "more workers go on after these pushes than one aggregated apply can serve (" +
                                        std::to_string(DSSPK_APPLY_MANY_MAX_DST) + "): push them in smaller groups");
        }
        if (d.ok) snap_worker[n_snap++] = workers[j];
        for (int e = 0; e < d.n_released; ++e) snap_worker[n_snap++] = released_out[n_rel + e];
        n_rel += d.n_released;
        for (int e = first; e < n_snap; ++e) {
            snap_after[e] = j + 1;
            pulled_version_out[snap_worker[e]] = c->version;
        }
    }
    if (c->host_only) return DSSP_OK;
    auto undo = [&](int rc) { restore_state(c, before); return rc; };
    const bool own = c->server_stream == nullptr;
    hipStream_t as = own ? c->wstream[workers[0]] : c->server_stream;
    for (int j = 0; j < m; ++j) {
        hipStream_t ws = c->wstream[workers[j]];
        if (ws == as) continue;
        if (hipEventRecord(c->ev_grad[workers[j]], ws) != hipSuccess || hipStreamWaitEvent(as, c->ev_grad[workers[j]], 0) != hipSuccess)
            return undo(fail(c, DSSP_EHIP, "event between a pusher's stream and the apply's"));
    }
    if (int rc = wait_for_w(c, as, before.version)) return undo(rc);
    float* dst[DSSPK_APPLY_MANY_MAX_DST];
    uint64_t* dst_stamp[DSSPK_APPLY_MANY_MAX_DST];
    for (int e = 0; e < n_snap; ++e) {
        dst[e] = pull_dst_dev[snap_worker[e]];
        if (!dst[e]) return undo(fail(c, DSSP_EINVAL, "pull_dst_dev of a worker that may go on is null"));
        if (int rc = ensure_stream(c, snap_worker[e])) return undo(rc);
        dst_stamp[e] = c->stamps_dev + 1 + snap_worker[e];
    }
    if (int rc = dsspk_apply_many(as, c->params, m, grads_dev, c->n_params, c->scale, n_snap, dst, snap_after, dst_stamp, c->stamps_dev,
                                  before.version + 1))
        return undo(fail(c, DSSP_EHIP, "aggregated apply kernel launch failed (rc " + std::to_string(rc) + ")"));
    HIP_TRY(c, hipEventRecord(c->ev_apply, as));
    for (int e = 0; e < n_snap; ++e)        // whoever got a snapshot goes on behind the kernel that wrote it
        if (c->wstream[snap_worker[e]] != as) HIP_TRY(c, hipStreamWaitEvent(c->wstream[snap_worker[e]], c->ev_apply, 0));
    return DSSP_OK;
}

namespace {

int ensure_wallclock(dssp_ctx* c, hipStream_t s) {
    if (c->ticks_host) return DSSP_OK;
    int dev = 0;
    HIP_TRY(c, hipGetDevice(&dev));
    HIP_TRY(c, hipDeviceGetAttribute(&c->wall_khz, hipDeviceAttributeWallClockRate, dev));
    if (c->wall_khz <= 0) return fail(c, DSSP_EHIP, "the device reports no wall clock rate");
    uint64_t* host = nullptr;
    HIP_TRY(c, hipHostMalloc((void**)&host, sizeof(uint64_t) * 4 * c->K, hipHostMallocDefault));
    for (int i = 0; i < 4 * c->K; ++i) host[i] = 0;
    void* devp = nullptr;
    hipError_t e = hipHostGetDevicePointer(&devp, host, 0);
    c->ev_done.assign(c->K, nullptr);
    for (int p = 0; p < c->K && e == hipSuccess; ++p) e = hipEventCreateWithFlags(&c->ev_done[p], hipEventDisableTiming);
    // time 0: the device clock now, read once through this stream
    if (e == hipSuccess && dsspk_clock_stamp(s, (uint64_t*)devp, nullptr) != 0) e = hipErrorLaunchFailure;
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        for (hipEvent_t ev : c->ev_done) if (ev) (void)hipEventDestroy(ev);
        c->ev_done.clear();
        (void)hipHostFree(host);
        return fail(c, DSSP_EHIP, std::string("wall-clock set-up: ") + hipGetErrorString(e));
    }
    c->origin_tick = host[0];
    host[0] = 0;
    c->timed_pending.assign(c->K, 0);
    c->ticks_host = host;
    c->ticks_dev = (uint64_t*)devp;
    return DSSP_OK;
}

int64_t ticks_to_us(const dssp_ctx* c, uint64_t tick) {
    const uint64_t dt = tick > c->origin_tick ? tick - c->origin_tick : 0;
    return (int64_t)(dt / (uint64_t)c->wall_khz * 1000 + dt % (uint64_t)c->wall_khz * 1000 / (uint64_t)c->wall_khz);
}

}  // namespace

extern "C" int dssp_worker_step_timed(dssp_ctx* c, int worker, const float* x_dev, const int32_t* y_dev, const float* w_local_dev,
                                      float* grad_dev, float* loss_dev, int slowdown_permille) {
    if (int rc = check_worker(c, worker)) return rc;
    if (c->host_only || !c->plan) return fail(c, DSSP_ESTATE, "worker_step before set_model");
    if (slowdown_permille < 1000 || slowdown_permille > 100000) return fail(c, DSSP_EINVAL, "slowdown_permille must be in [1000, 100000]");
    if (int rc = ensure_stream(c, worker)) return rc;
    hipStream_t s = c->wstream[worker];
    if (int rc = ensure_wallclock(c, s)) return rc;
    if (c->timed_pending[worker]) return fail(c, DSSP_ESTATE, "the worker's previous timed step was not collected with dssp_step_done");
    uint64_t* slot = c->ticks_dev + 4 * worker;
    if (dsspk_clock_stamp(s, slot, nullptr)) return fail(c, DSSP_EHIP, "clock stamp launch failed");
    if (int rc = dssp_worker_step(c, worker, x_dev, y_dev, w_local_dev, grad_dev, loss_dev)) return rc;
    // at most 0.1 s of extra time per iteration
    if (dsspk_clock_stretch(s, slot, slowdown_permille, (uint64_t)c->wall_khz * 100, slot + 1, slot + 2))
        return fail(c, DSSP_EHIP, "clock stretch launch failed");
    HIP_TRY(c, hipEventRecord(c->ev_done[worker], s));
    c->timed_pending[worker] = 1;
    return DSSP_OK;
}

extern "C" int dssp_step_done(dssp_ctx* c, int worker, int* done_out, int64_t* t_start_us_out, int64_t* t_gradient_us_out,
                              int64_t* t_done_us_out) {
    if (int rc = check_worker(c, worker)) return rc;
    if (!done_out) return fail(c, DSSP_EINVAL, "null output pointer");
    if (!c->ticks_host || !c->timed_pending[worker]) return fail(c, DSSP_ESTATE, "no timed step of this worker is under way");
    const hipError_t e = hipEventQuery(c->ev_done[worker]);
    if (e == hipErrorNotReady) { *done_out = 0; return DSSP_OK; }
    if (e != hipSuccess) return fail(c, DSSP_EHIP, std::string("hipEventQuery: ") + hipGetErrorString(e));
    const volatile uint64_t* slot = c->ticks_host + 4 * worker;
    *done_out = 1;
    if (t_start_us_out) *t_start_us_out = ticks_to_us(c, slot[0]);
    if (t_gradient_us_out) *t_gradient_us_out = ticks_to_us(c, slot[1]);
    if (t_done_us_out) *t_done_us_out = ticks_to_us(c, slot[2]);
    c->timed_pending[worker] = 0;
    return DSSP_OK;
}

extern "C" int dssp_clock(dssp_ctx* c, int64_t* t_out, int32_t* r_out, uint8_t* blocked_out, uint64_t* version_out) {
    if (!c) return DSSP_EINVAL;
    for (int i = 0; i < c->K; ++i) {
        if (t_out) t_out[i] = c->t[i];
        if (r_out) r_out[i] = c->r[i];
        if (blocked_out) blocked_out[i] = c->blocked[i];
    }
    if (version_out) *version_out = c->version;
    return DSSP_OK;
}

extern "C" int dssp_synchronize(dssp_ctx* c) {
    if (!c) return DSSP_EINVAL;
    if (c->host_only) return DSSP_OK;
    if (c->server_stream) HIP_TRY(c, hipStreamSynchronize(c->server_stream));
    for (int p = 0; p < c->K; ++p)
        if (c->wstream[p]) HIP_TRY(c, hipStreamSynchronize(c->wstream[p]));
    return DSSP_OK;
}

extern "C" int dssp_device_stamps(dssp_ctx* c, uint64_t* stamps_out) {
    if (!c || !stamps_out) return DSSP_EINVAL;
    if (c->host_only) return fail(c, DSSP_ESTATE, "host-only context has no device stamps");
    if (int rc = dssp_synchronize(c)) return rc;
    HIP_TRY(c, hipMemcpy(stamps_out, c->stamps_dev, sizeof(uint64_t) * (c->K + 1), hipMemcpyDeviceToHost));
    return DSSP_OK;
}

extern "C" const char* dssp_last_error(dssp_ctx* c) { return c ? c->err.c_str() : "null context"; }

extern "C" int dssp_destroy(dssp_ctx* c) {
    if (!c) return DSSP_EINVAL;
    if (!c->host_only) {
        if (c->server_stream) (void)hipStreamSynchronize(c->server_stream);
        for (int p = 0; p < c->K; ++p)
            if (c->wstream[p]) (void)hipStreamSynchronize(c->wstream[p]);
        drop_step_graphs(c);
        if (c->plan) dssp_model::destroy(c->plan);
        if (c->ev_apply) (void)hipEventDestroy(c->ev_apply);
        for (int p = 0; p < c->K; ++p) {
            if (c->ev_grad[p]) (void)hipEventDestroy(c->ev_grad[p]);
            if (c->ev_pull[p]) (void)hipEventDestroy(c->ev_pull[p]);
            if (c->own_wstream[p] && c->wstream[p]) (void)hipStreamDestroy(c->wstream[p]);
        }
        if (c->stamps_dev) (void)hipFree(c->stamps_dev);
        for (hipEvent_t ev : c->ev_done) if (ev) (void)hipEventDestroy(ev);
        if (c->ticks_host) (void)hipHostFree(c->ticks_host);
    }
    delete c;
    return DSSP_OK;
}
