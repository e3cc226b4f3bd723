/* libdssp: Dynamic Stale Synchronous Parallel parameter-server training, hot path,
 * K virtual workers on HIP streams of one MI355X (gfx950).
 *
 * The calls follow the paper's problem statement (Sec. III-A) and Algorithm 1:
 *   worker part : wait for OK, pull w, replace local weights, gradient of the
 *                 mini-batch loss on the local weights, push the gradient;
 *   server part : count the push, apply the gradient to the global weights,
 *                 decide OK-now or wait (credit r_p, lower bound s_L, the
 *                 synchronization controller of Algorithm 2 for the fastest worker).
 *
 * General rules
 *  - All pointers named *_dev are DEVICE pointers owned by the caller and only
 *    borrowed for the duration documented per call; all others are HOST pointers.
 *    Parameter, gradient, snapshot and image buffers must be 16-byte aligned (the
 *    kernels move 16-byte vectors); a misaligned buffer is rejected with DSSP_EHIP.
 *  - Every call returns DSSP_OK (0) or a negative error code; nothing throws.
 *    dssp_last_error() gives a readable message for the last failing call on that
 *    context (valid until the next call on it).
 *  - Calls are asynchronous with respect to the device: they enqueue work on the
 *    worker's / server's stream and never synchronise the device.  Host-visible
 *    outputs (ok, released, clocks, versions) are decided on the host and valid on
 *    return.  A context must be used from one host thread at a time.
 *  - Time is virtual: timestamps are int64 ticks supplied by the caller.
 *
 * Layouts (fp32 everywhere)
 *  - images            x[m][32][32][3]          (channels last)
 *  - labels            y[m] int32 in [0, n_classes)
 *  - flat parameter / gradient vector: layers in forward order; convolution
 *    filter [KH][KW][Cin][Cout] then bias [Cout] if the layer has one; batch norm
 *    gamma[C] then beta[C]; fully connected weight [in][out] then bias [out].
 *    A feature map is flattened in (h, w, c) order in front of the first fully
 *    connected layer.  dssp_model_segments() reports the segments.
 */
#ifndef DSSP_H
#define DSSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dssp_ctx dssp_ctx;

enum {
    DSSP_OK = 0,
    DSSP_EINVAL = -1,   /* bad argument: null pointer, worker out of range, K < 1, s_L < 0, r_max < 0, ... */
    DSSP_ESTATE = -2,   /* call not legal now: push / pull by a worker that is waiting for OK (the answer to its last
                           push was "wait" and no later push has released it), worker_step before set_model, ... */
    DSSP_EHIP = -3,     /* a HIP runtime call failed; text in dssp_last_error() */
    DSSP_ENOMEM = -4    /* workspace too small */
};

/* model_id for dssp_set_model and the dssp_model_* queries.  Any 6n+2 >= 8 selects
 * the CIFAR ResNet of that depth (8, 20, 50, 56, 110, ...). */
enum {
    DSSP_MODEL_NONE = 0,        /* flat vector only: push / pull / clock, no worker_step */
    DSSP_MODEL_MLP = 1,         /* 3072 - 256 - n_classes, ReLU */
    DSSP_MODEL_ALEXNET_DS = 2,  /* conv5x5x64, maxpool3s2, conv5x5x64, maxpool3s2, FC384, FC192, FC n_classes */
    DSSP_MODEL_ALEXNET_3C = 3,  /* Sec. V-A3's reduced AlexNet, three convolutional and two fully connected layers (widths:
                                   this library's reading): conv5x5x64, maxpool3s2, conv5x5x64, maxpool3s2, conv3x3x64,
                                   FC384, FC n_classes */
    DSSP_MODEL_RESNET110 = 110  /* 3 stages x 18 basic blocks, 16/32/64 channels, BN, parameter-free shortcuts */
};

#define DSSP_S_L_NEVER_WAIT 2147483647   /* s_L of the asynchronous paradigm (Sec. I-A2): nobody ever waits */

/* Problem statement, Sec. III-A: lower bound s_L and range R = [0, r_max] (s_U = s_L + r_max).
 * (s_L, r_max) = (0, 0) is BSP, (s, 0) is SSP with threshold s, s_L = DSSP_S_L_NEVER_WAIT is ASP
 * (Sec. I-A).  The server applies w <- w - (lr / K) * g per push (Alg. 1, server step 2).
 *   out         receives the context
 *   params_dev  global weights w, n_params floats, caller-owned, updated in place by pushes.
 *               params_dev == NULL with n_params == 0 creates a host-only context: the
 *               decision logic runs, no device work is enqueued and no HIP call is made.
 * All workers start with OK granted (they may pull version 0 and start iteration 1). */
int dssp_create(dssp_ctx** out, float* params_dev, int64_t n_params,
                int K, int s_L, int r_max, float lr);

/* Streams: worker in [0, K), or -1 for a stream of the server's own.  hip_stream is a
 * hipStream_t created by the caller (default priority); it must outlive the context.
 * Worker streams the caller did not set - and a worker's stream given as NULL, the legacy default stream, which this
 * library never enqueues on - are created by the context on first use (non-blocking, default priority) and owned by
 * it; work the caller has on the default stream is NOT ordered with them: order it with dssp_synchronize or events.  The server
 * has no stream unless one is set: each apply then runs on the pusher's stream, right behind
 * the gradient it consumes, and the context's events keep applies in push order and behind
 * every snapshot still being read.  With a server stream (nullptr takes it away again) the
 * applies run there instead, behind the same events; results are identical, but a stream
 * that shares a hardware queue with a worker's stream makes the small apply wait for that
 * worker's whole iteration. */
int dssp_set_stream(dssp_ctx* ctx, int worker, void* hip_stream);

/* Which of n idle streams share a hardware queue (no passage of the paper: a property of the
 * device runtime that decides how K workers on one GPU should be dealt onto streams).  A process
 * has few hardware queues and the runtime spreads streams over them unevenly; work on streams of
 * one queue runs one after the other, so workers should sit on streams of different queues, the
 * same number on each.  queue_out[i] receives the queue number of hip_streams[i], numbered from 0
 * in order of first appearance; n_queues_out (may be NULL) the number of queues seen.  Measured,
 * not looked up: for each pair tested a kernel spins for 2 ms on one stream while a kernel on the
 * other reads the device clock, so the call takes up to about n * queues * 4 ms and synchronises the given
 * streams.  n in [1, 64]; the current device is used; needs no context.  Returns DSSP_EINVAL or
 * DSSP_EHIP on failure. */
int dssp_stream_queues(void* const* hip_streams, int n, int* queue_out, int* n_queues_out);

/* Selects the network of dssp_worker_step and hands over scratch memory.
 *   workspace_dev    at least dssp_workspace_bytes(...) bytes, 256-byte aligned, caller-owned,
 *                    used by the library until dssp_destroy (activations saved for backward,
 *                    partial sums); contents are undefined between calls.
 * n_params given to dssp_create must equal dssp_model_param_count(model_id, n_classes). */
int dssp_set_model(dssp_ctx* ctx, int model_id, int batch, int n_classes,
                   void* workspace_dev, size_t workspace_bytes);

/* Alg. 1, worker steps 2-3: copy the global weights into the worker's local weights.
 * Legal only when the worker holds an OK (initially, after a push answered ok, or after it was
 * released).  Enqueued on the worker's stream behind the apply of every push decided so far;
 * later applies wait for this copy.
 *   dst_dev      n_params floats
 *   version_out  (host, may be NULL) number of applies contained in the snapshot */
int dssp_pull(dssp_ctx* ctx, int worker, float* dst_dev, uint64_t* version_out);

/* Alg. 1, worker step 4: g = (1/m) sum_i d loss((x_i, y_i), w_local) / dw, loss = softmax
 * cross-entropy of the network selected by dssp_set_model.  Enqueued on the worker's stream.
 *   x_dev [m][32][32][3], y_dev [m], w_local_dev / grad_dev n_params floats (grad is overwritten),
 *   loss_dev  1 float, mean loss of the mini-batch (may be NULL).
 * The launch sequence depends only on (worker, the five pointers): its second use with the same
 * pointers is captured into a HIP graph and replayed from then on, so callers should cycle through a
 * fixed set of buffers.  Setting the environment variable DSSP_NO_GRAPH=1 before dssp_create keeps
 * every step as individual launches. */
int dssp_worker_step(dssp_ctx* ctx, int worker, const float* x_dev, const int32_t* y_dev,
                     const float* w_local_dev, float* grad_dev, float* loss_dev);

/* Alg. 1, worker step 5 + server part, Alg. 2: the push of `worker` reaches the server at
 * virtual time t_push_ticks.  Counts it, decides, and enqueues the apply behind the worker's
 * gradient computation (on the worker's stream, or on the server's if one was set).
 *   grad_dev         n_params floats; must stay untouched until the worker's next pull has run
 *                    (the next dssp_worker_step of that worker may overwrite it)
 *   ok_out           1 = OK now, 0 = the worker waits until a later push releases it
 *   released_out     [K] indices of workers released by this push, ascending
 *   n_released_out   how many
 *   rstar_out        (may be NULL) r* returned by the synchronization controller, -1 if not called
 *   grant_out        (may be NULL) extra iterations actually granted (r* capped so that the gap
 *                    never exceeds s_L + r_max), -1 if the controller was not called */
int dssp_push(dssp_ctx* ctx, int worker, const float* grad_dev, int64_t t_push_ticks,
              int* ok_out, int* released_out, int* n_released_out, int* rstar_out, int* grant_out);

/* dssp_push whose apply also serves as the pusher's next pull when the pusher is granted OK at once (Alg. 1, server
 * step 2 and worker steps 2-3 in one pass over the weights: 16 instead of 20 bytes per parameter).  Decisions,
 * counters and results are those of dssp_push followed by dssp_pull(worker, pull_dst_dev).
 *   pull_dst_dev     where the pusher's snapshot goes (n_params floats, 16-byte aligned; ignored by a host-only context)
 *   pulled_out       1 = the snapshot of version *version_out has been enqueued into pull_dst_dev: the worker goes
 *                    straight to its next dssp_worker_step; 0 = the worker was blocked, only the apply was enqueued,
 *                    and it pulls with dssp_pull once a later push releases it
 *   version_out      (may be NULL) number of applies including this one */
int dssp_push_pull(dssp_ctx* ctx, int worker, const float* grad_dev, int64_t t_push_ticks, float* pull_dst_dev,
                   int* ok_out, int* released_out, int* n_released_out, int* rstar_out, int* grant_out,
                   int* pulled_out, uint64_t* version_out);

/* Alg. 1, server step 2, for pushes that arrive together: "if some other workers send their updates at the same
 * time, their gradients are aggregated before updating".  m workers push at the same virtual time t_push_ticks.  The
 * pushes are still counted and decided one at a time, in ascending worker order, exactly as m calls of dssp_push_pull
 * would (every decision sees the clocks left by the pushes before it); what is aggregated is the device work: ONE
 * kernel reads the weights once, takes in the m gradients in that order and writes the weights once, and every worker
 * that may go on after push j - its pusher if answered OK, the workers that push releases - receives the weights as
 * they are after push j in its snapshot, from the same pass.  Weights, snapshots and stamps are bit-identical to the m
 * single calls; the traffic is (4 m + 8 + 4 snapshots) bytes per parameter instead of 12 m + 8 snapshots.
 *   workers           [m] distinct, ascending; m in [1, 16]; none of them waiting for OK
 *   grads_dev         [m] host array of device pointers, n_params floats each; untouched until that worker's next step
 *   pull_dst_dev      [K] host array: where worker q's snapshot goes (device, n_params floats, 16-byte aligned), for
 *                     every worker that can go on (all K to be safe); ignored by a host-only context
 *   ok_out            [m] answer to each push;  rstar_out, grant_out [m] as in dssp_push (may be NULL)
 *   n_released_out    [m] how many workers push j released;  released_out [K] their indices, push after push
 *   pulled_version_out [K] version of the snapshot enqueued for worker q by this call, 0 if none: such a worker goes
 *                     straight to its next dssp_worker_step (no dssp_pull)
 * DSSP_EINVAL if more than 32 workers would have to be served by the one kernel (push smaller groups).  On any error
 * nothing has been counted. */
int dssp_push_many(dssp_ctx* ctx, int m, const int* workers, const float* const* grads_dev, int64_t t_push_ticks,
                   float* const* pull_dst_dev, int* ok_out, int* rstar_out, int* grant_out, int* n_released_out,
                   int* released_out, uint64_t* pulled_version_out);

/* Wall-clock mode: Alg. 2's input is the real time at which a push reaches the server, and Sec. V-C runs on GPUs of
 * unequal speed.  dssp_worker_step_timed is dssp_worker_step bracketed by reads of the GPU's constant-rate clock on
 * the worker's stream, followed by a hold that keeps the stream busy until the iteration has lasted
 * slowdown_permille / 1000 times what it really took (1000: no hold; at most 0.1 s extra): the worker behaves like one
 * on a GPU that much slower.  dssp_step_done polls, without blocking, whether that iteration (hold included) has left
 * the stream; if so it reports, in microseconds of device time since the context's first timed step, when the
 * iteration started, when its gradient was complete and when the hold ended - the last is the timestamp to hand to
 * dssp_push.  One timed step per worker at a time (DSSP_ESTATE otherwise).  Pinned host memory for the clock values
 * is allocated on first use. */
int dssp_worker_step_timed(dssp_ctx* ctx, int worker, const float* x_dev, const int32_t* y_dev,
                           const float* w_local_dev, float* grad_dev, float* loss_dev, int slowdown_permille);
int dssp_step_done(dssp_ctx* ctx, int worker, int* done_out, int64_t* t_start_us_out, int64_t* t_gradient_us_out,
                   int64_t* t_done_us_out);

/* Read-only view of the server's counters (Alg. 1 preamble): t[K] pushes received,
 * r[K] remaining extra-iteration credit, blocked[K] 1 while waiting for OK, version = number
 * of applies.  Any output may be NULL. */
int dssp_clock(dssp_ctx* ctx, int64_t* t_out, int32_t* r_out, uint8_t* blocked_out,
               uint64_t* version_out);

/* Version stamps as the DEVICE saw them: stamps_out[0] = stamp written by the last apply,
 * stamps_out[1 + p] = stamp copied by worker p's last pull.  Synchronises all streams of the
 * context (a diagnostic: it detects a pull that ran out of order with an apply). */
int dssp_device_stamps(dssp_ctx* ctx, uint64_t* stamps_out /* [K + 1] */);

/* Blocks the host until everything enqueued on the context's streams has finished. */
int dssp_synchronize(dssp_ctx* ctx);

const char* dssp_last_error(dssp_ctx* ctx);
int dssp_destroy(dssp_ctx* ctx);

/* Host-only queries (no GPU needed). */
int64_t dssp_model_param_count(int model_id, int n_classes);            /* < 0: unknown model */
/* kind: 0 weight, 1 bias, 2 BN gamma, 3 BN beta.  fan_in: inputs per output unit (weights only).
 * Returns the number of segments (also when max_segments is smaller; nothing is written past it). */
int dssp_model_segments(int model_id, int n_classes, int32_t* kind, int64_t* size, int64_t* fan_in,
                        int max_segments);
size_t dssp_workspace_bytes(int model_id, int batch, int n_classes, int K);
/* Where worker p's saved post-ReLU activation / max-pool choice number `index` (forward order)
 * lives inside the workspace: byte offset and element count.  what: 0 = ReLU output (float),
 * 1 = max-pool choice (uint8 window position kh*3+kw), 2 = logits (float).  Returns DSSP_EINVAL
 * past the last one.  For tests that check the discrete decisions of a step. */
int dssp_workspace_tensor(int model_id, int batch, int n_classes, int K, int worker, int what, int index,
                          size_t* byte_offset, int64_t* count);

#ifdef __cplusplus
}
#endif
#endif
