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

// Alg. 2 from step 3 on (table A was shifted when the push arrived).  Extrapolates r_max+1 push
// times of p (from its current push) and of the slowest worker (from one interval after its latest
// push) and returns the index on p's timeline that comes closest to any push of the slowest worker.
int synchronization_controller(const dssp_ctx* c, int p) {
    const int slow = find_slowest(c);
    const int64_t ip = c->A[p][0] - c->A[p][1];
    const int64_t is = c->A[slow][0] - c->A[slow][1];
    int r_star = 0;
    bool have = false;
    __int128 best = 0;
    for (int rr = 0; rr <= c->r_max; ++rr) {
        const __int128 sp = (__int128)c->A[p][0] + (__int128)rr * ip;
        for (int k = 0; k <= c->r_max; ++k) {
            const __int128 ss = (__int128)c->A[slow][0] + (__int128)(k + 1) * is;
            const __int128 d = ss > sp ? ss - sp : sp - ss;
            if (!have || d < best) { have = true; best = d; r_star = rr; }
        }
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
        sg->graph = graph;
        HIP_TRY(c, hipGraphInstantiate(&sg->exec, graph, nullptr, nullptr, 0));
        HIP_TRY(c, hipGraphLaunch(sg->exec, s));
        return DSSP_OK;
    }
    if (rc) return fail(c, DSSP_EHIP, "worker_step: " + err + " (rc " + std::to_string(rc) + ")");
    if (sg) sg->calls += 1;
    return DSSP_OK;
}

// Alg. 1 server part for one push.  The decision (steps 3-16 and Alg. 2) is integer work on the host and does not
// depend on the apply, so it is taken first; the device work enqueued afterwards is the apply alone, or - if the
// pusher may go on at once and handed over where its next snapshot goes - apply and pull in one kernel.
static int push_impl(dssp_ctx* c, int worker, const float* grad_dev, int64_t t_push, float* pull_dst_dev, int* ok_out,
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
    // Alg. 2 steps 1-2, done for every push so that A really holds the two latest pushes of all workers
    c->A[p][1] = c->A[p][0];
    c->A[p][0] = t_push;
    c->t[p] += 1;            // Alg. 1 server step 1
    c->version += 1;         // Alg. 1 server step 2 (the apply enqueued below)
    int r_star = -1, grant = -1;
    bool ok;
    if (c->r[p] > 0) {       // steps 3-5: spend one unit of credit
        c->r[p] -= 1;
        ok = true;
    } else {
        const int64_t t_min = *std::min_element(c->t.begin(), c->t.end());
        const int64_t t_max = *std::max_element(c->t.begin(), c->t.end());
        const int64_t gap = c->t[p] - t_min;
        if (gap <= c->s_L) {
            ok = true;       // steps 8-9
        } else if (c->t[p] == t_max) {
            r_star = synchronization_controller(c, p);                        // step 12
            const int64_t room = (int64_t)c->s_L + c->r_max - gap + 1;        // keeps the gap <= s_L + r_max
            grant = (int)std::min<int64_t>(r_star, room);
            if (grant >= 1) { c->r[p] = grant - 1; ok = true; }               // this OK is the first extra iteration
            else ok = false;
        } else {
            ok = false;      // step 16: wait for the slowest worker
        }
    }
    c->has_ok[p] = ok ? 1 : 0;
    c->blocked[p] = ok ? 0 : 1;
    int n_rel = 0;
    const int64_t t_min = *std::min_element(c->t.begin(), c->t.end());
    for (int q = 0; q < c->K; ++q)
        if (q != p && c->blocked[q] && c->t[q] - t_min <= c->s_L) {
            c->blocked[q] = 0;
            c->has_ok[q] = 1;
            released_out[n_rel++] = q;
        }
    const bool fused = ok && pull_dst_dev != nullptr;
    if (!c->host_only) {
        // The apply runs behind the worker's gradient, behind the apply before it and behind every snapshot still
        // reading w.  Without a server stream it goes onto the pusher's own stream, right behind the gradient: a
        // separate stream shares a hardware queue with some worker's stream, and the small apply then waits for
        // that worker's whole iteration.
        const bool own = c->server_stream == nullptr;
        hipStream_t as = own ? c->wstream[p] : c->server_stream;
        if (!own) {
            HIP_TRY(c, hipEventRecord(c->ev_grad[p], c->wstream[p]));
            HIP_TRY(c, hipStreamWaitEvent(as, c->ev_grad[p], 0));
        }
        if (c->version > 1) HIP_TRY(c, hipStreamWaitEvent(as, c->ev_apply, 0));
        for (int q = 0; q < c->K; ++q)
            if (c->pull_pending[q]) {
                if (c->wstream[q] != as) HIP_TRY(c, hipStreamWaitEvent(as, c->ev_pull[q], 0));
                c->pull_pending[q] = 0;
            }
        int rc;
        if (fused)      // the worker's stream gets at the snapshot through ev_apply, like at any other pull
            rc = dsspk_apply_pull(as, c->params, grad_dev, pull_dst_dev, c->n_params, c->scale, c->stamps_dev,
                                  c->stamps_dev + 1 + p, c->version);
        else
            rc = dsspk_apply(as, c->params, grad_dev, c->n_params, c->scale, c->stamps_dev, c->version);
        if (rc) return fail(c, DSSP_EHIP, "apply kernel launch failed (rc " + std::to_string(rc) + ")");
        HIP_TRY(c, hipEventRecord(c->ev_apply, as));
        if (fused && !own) HIP_TRY(c, hipStreamWaitEvent(c->wstream[p], c->ev_apply, 0));
    }
    *ok_out = ok ? 1 : 0;
    *n_released_out = n_rel;
    if (rstar_out) *rstar_out = r_star;
    if (grant_out) *grant_out = grant;
    if (pulled_out) *pulled_out = fused ? 1 : 0;
    if (version_out) *version_out = c->version;
    return DSSP_OK;
}

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
    }
    delete c;
    return DSSP_OK;
}
