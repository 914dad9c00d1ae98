/*
 * pooch.h -- C ABI of the MI355X out-of-core CNN training step.
 *
 * One training step (forward + backward propagation, paper section 2.1) of a CNN is run
 * inside a caller-supplied device arena whose size IS the memory budget.  Every feature
 * map that some backward computation needs is handled in one of three ways (section
 * 4.1.1): kept resident, swapped to pinned host memory after its last forward use and
 * brought back before backward needs it (section 3.1), or discarded and recomputed from
 * its producer's inputs, recursively (section 3.2).  The per-map class ("plan") comes from
 * the paper's three phases (section 4.1.2): profile -> classify -> execute.
 *
 * Conventions
 *   - plain C, no exceptions cross the boundary; every call returns a status (or an id >= 0
 *     / a negative status).  pooch_last_error() gives the text of the last failure.
 *   - HOST pointers unless a parameter is marked DEVICE.  Host tensors are fp32 in the
 *     logical layout NC(D)HW / KC(kd)(kh)(kw), row-major; the library converts to its own
 *     device layout (channels-last) on the way in and back on the way out.
 *   - The caller owns the arena, the pinned buffer and the three streams (typically a
 *     torch uint8 CUDA tensor, a pinned torch tensor, torch streams).  The library never
 *     allocates device memory for tensors: parameters, gradients, batch statistics,
 *     workspaces, the input batch, every activation and every gradient map live at
 *     offsets inside the arena, so exceeding the budget is impossible by construction.
 *     Running out of room is a PLANNING-time error (POOCH_E_BUDGET), never a mid-step one:
 *     plans that run out of memory are excluded when the plan is made (section 4.1.1).
 *   - A context is not thread-safe; use one per thread.  All streams must have default
 *     priority.
 *   - A context created with arena == NULL is "planning only": graph, profile injection,
 *     planning and simulation work (no GPU needed), compute calls return POOCH_E_STATE.
 *   - Two environment variables switch kernel paths off for A/B measurements (results stay
 *     within rounding): POOCH_NO_CONV_STATS (read by pooch_finalize: batch normalisations take
 *     their own statistics pass), POOCH_NO_LINEAR (read at the first convolution launch: the
 *     convolution kernels recompute every tile address from scratch).
 */
#ifndef POOCH_H
#define POOCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pooch_ctx pooch_ctx;
typedef int32_t pooch_status;

enum {
    POOCH_OK = 0,
    POOCH_E_INVALID = -1,   /* bad argument / malformed graph */
    POOCH_E_STATE = -2,     /* call out of order (e.g. step before a plan exists) */
    POOCH_E_BUDGET = -3,    /* the plan (or any plan) does not fit the arena / pinned buffer */
    POOCH_E_HIP = -4,       /* a HIP runtime call failed */
    POOCH_E_NOPROFILE = -5  /* planning needs a profile and none was measured or injected */
};

/* classes of a feature map, section 4.1.1 */
enum { POOCH_KEEP = 0, POOCH_SWAP = 1, POOCH_RECOMPUTE = 2 };

/* planning modes: in-core (everything kept), the four methods compared in section 5.1, one extension, and the
 * static policy of section 5.2 */
enum {
    POOCH_MODE_INCORE = 0,
    POOCH_MODE_SWAPALL_NOSCHED = 1, /* all swap; each swap-in starts with the previous backward computation */
    POOCH_MODE_SWAPALL = 2,         /* all swap; swap-ins moved up as far as memory allows (section 4.3) */
    POOCH_MODE_SWAPOPT = 3,         /* keep/swap search only (section 4.4.2) */
    POOCH_MODE_POOCH = 4,           /* keep/swap search, then swap/recompute classification (section 4.4.3) */
    POOCH_MODE_REFINE = 5,          /* not in the paper: POOCH followed by an iterated local search over single class
                                       changes, judged by the same timeline simulation.  If the profile has been
                                       replaced or refined since the installed plan was made, that plan competes
                                       with the two-step plan as the search's starting point (the faster one by
                                       simulation under the current profile is taken) */
    POOCH_MODE_SUPERNEURONS = 6     /* the static policy section 5.2 compares against: keep from the output layer while
                                       it fits, then convolution outputs swap and the rest is recomputed; swap-ins
                                       are not moved up */
};

/* ---- context ------------------------------------------------------------------------
 * arena        DEVICE pointer, 256-byte aligned, arena_bytes long (== the budget); may be
 *              NULL for a planning-only context (arena_bytes still sets the budget).  The budget
 *              counts in whole 256-byte units: a tail of arena_bytes % 256 bytes is never used.
 * pinned_host  pinned HOST buffer that receives swapped-out maps; may be NULL/0 when no
 *              plan ever swaps.
 * stream_*     hipStream_t handles passed as void*: compute, device-to-host, host-to-device.
 *              Three distinct streams give overlap; passing the same stream is legal.  Distinct is not
 *              enough for overlap: the runtime maps streams onto a few hardware queues (four by default),
 *              and two streams on one queue run their work in order -- a swap copy then sits in front of
 *              kernels.  Create the three one right after the other (hipStreamCreateWithFlags), as the Python
 *              binding does; streams picked from a pool that has served many earlier contexts were seen to
 *              collide (ResNet-50, batch 640: the step 30 % slower).  Default priority only.
 * The context borrows all five; they must outlive it.  */
pooch_status pooch_create(void *arena, size_t arena_bytes, void *pinned_host, size_t pinned_bytes,
                          void *stream_compute, void *stream_d2h, void *stream_h2d, pooch_ctx **out);
void pooch_destroy(pooch_ctx *);
const char *pooch_last_error(pooch_ctx *);

/* ---- graph (section 4.2: "computation graph and dependency of the NN") ----------------
 * Insertion order is execution order.  Each call returns the id (>= 0) of the tensor the
 * layer produces, or a negative status.  nspatial is 2 or 3; k/stride/pad have nspatial
 * entries ordered (d,)h,w.  dims of the input are N,C,(D,)H,W.
 * conv: cross-correlation, zero padding, no bias.  bn: training-mode batch normalisation
 * over batch x space with learnable gamma/beta.  maxpool pads with -inf and sends the
 * gradient to the first maximal element in scan order.  fc has a bias.  add takes two
 * different tensors of one shape (a + a is POOCH_E_INVALID).  softmax_ce is the
 * terminal node: mean over the batch of the softmax cross-entropy against int32 labels. */
int32_t pooch_input(pooch_ctx *, const int64_t *dims, int ndim);
int32_t pooch_conv(pooch_ctx *, int32_t x, int cout, const int *k, const int *stride, const int *pad, int nspatial);
int32_t pooch_bn(pooch_ctx *, int32_t x, float eps);
int32_t pooch_relu(pooch_ctx *, int32_t x);
int32_t pooch_add(pooch_ctx *, int32_t a, int32_t b);
int32_t pooch_maxpool(pooch_ctx *, int32_t x, const int *k, const int *stride, const int *pad, int nspatial);
int32_t pooch_gavgpool(pooch_ctx *, int32_t x);
int32_t pooch_fc(pooch_ctx *, int32_t x, int nout);
int32_t pooch_softmax_ce(pooch_ctx *, int32_t logits);
/* Layer fusion (default on; call before pooch_finalize): a bn or add whose only consumer is a
 * relu is executed inside that relu, so its output is never written to memory.  Results are
 * those of the unfused layers; the feature-map set is unchanged (backward of a fused bn+relu
 * reads the bn's input and re-derives the relu decision from it).
 * A bn whose only consumer is the add of such an add + relu is applied inside that kernel as well
 * (either input of the add, or both): its forward step is the batch statistics alone, its output is
 * never written, its backward is unchanged.
 * pooch_node_fused: id of the relu a layer's output is produced in, -1 if the layer writes its own. */
pooch_status pooch_set_fusion(pooch_ctx *, int enable);
int32_t pooch_node_fused(pooch_ctx *, int32_t id);
/* One-bit ReLU masks (default off; call before pooch_finalize): a relu, or an add + relu, whose output no other
 * layer's backward reads -- the one in front of a global average pool, say -- keeps one bit per element ("was the
 * output positive") in the resident region for its own backward, which asks nothing else of the output.  The output
 * then is no feature map (section 4.1.1 classifies what some backward computation reads): it is freed after its last
 * forward consumer and never swapped or recomputed for the backward pass.  Results are bit-identical to those
 * without masks.  Off by default because it takes ResNet-50 from the 105 feature maps of table 3 to 104.
 * pooch_node_keeps_mask: 1 if layer `id` keeps such a mask, 0 if not. */
pooch_status pooch_set_relu_masks(pooch_ctx *, int enable);
int32_t pooch_node_keeps_mask(pooch_ctx *, int32_t id);
/* A convolution whose result goes directly into a batch normalisation also produces that
 * layer's batch statistics while its results are still on chip, which saves the normalisation
 * one of its three passes over the tensor (section 3.3 counts these layers as pure memory
 * traffic).  pooch_bn_stats_source: id of the conv that supplies layer `id`'s statistics in a
 * forward pass, -1 if the layer reads its input for them itself (also for ids that are no bn).
 * A re-forward in backward always re-applies the saved statistics. */
int32_t pooch_bn_stats_source(pooch_ctx *, int32_t id);
/* Freezes the graph: shapes, liveness, the feature-map list (every tensor some backward
 * reads, except the network input, which is caller data and stays resident), the parameter
 * list and the layout of the resident region at the bottom of the arena.
 * POOCH_E_BUDGET if the resident region alone exceeds the arena. */
pooch_status pooch_finalize(pooch_ctx *);

/* ---- parameters and data -------------------------------------------------------------
 * Parameters in layer order: conv -> W[K,C,k...]; bn -> gamma[C], beta[C]; fc -> W[O,I], b[O]
 * (I flattened in logical C,(D,)H,W order).  set_* copy from host synchronously; get_grad
 * copies the gradient of parameter i (same shape) back after a step.
 * Anything that runs the network (pooch_step, pooch_step_timed, the profiling calls) returns
 * POOCH_E_STATE until a batch and every parameter have been set (labels index the logits, so
 * stale memory must never be run); pooch_get_grad and pooch_sgd_update return POOCH_E_STATE
 * until a step has run. */
int32_t pooch_num_params(pooch_ctx *);
pooch_status pooch_param_info(pooch_ctx *, int32_t i, int64_t *numel, int32_t *node);
pooch_status pooch_set_param(pooch_ctx *, int32_t i, const float *host);
pooch_status pooch_get_grad(pooch_ctx *, int32_t i, float *host);
pooch_status pooch_set_batch(pooch_ctx *, const float *x_host, const int32_t *labels_host);
/* Plain SGD on every parameter with the gradients of the last step: p -= lr * grad (section 2.1's third
 * phase; the paper leaves it out of its timelines because it is short).  Synchronises.
 * pooch_get_param reads parameter i back in the layout pooch_set_param takes. */
pooch_status pooch_sgd_update(pooch_ctx *, float lr);
pooch_status pooch_get_param(pooch_ctx *, int32_t i, float *host);
/* parity aid: during every following step, right after the forward of layer `id` has run,
 * its output is copied to `host` in logical layout (the step synchronises there, so this is
 * for tests, not for timed runs).  host == NULL cancels the capture of that layer.  The
 * buffer must stay valid until cancelled or the context is destroyed. */
pooch_status pooch_capture_tensor(pooch_ctx *, int32_t id, float *host);
/* test aid for the error path: the next replay of a command list (pooch_step, pooch_step_timed, a profiling
 * iteration, pooch_refine_profile) reports POOCH_E_HIP when it reaches command `command_index` (a row of
 * pooch_get_commands for pooch_step) instead of enqueueing it, once; a negative index cancels.  Nothing faults: the
 * commands before it run normally.  What every failure inside a step guarantees, injected or real: the call returns
 * only after everything it had enqueued has finished; gradients count as absent until a later step completes;
 * parameters, batch, profile and plan are untouched, so the same context may step again (BN running averages of
 * the layers that ran have moved).  A failed profiling iteration drops the samples gathered so far. */
pooch_status pooch_inject_failure(pooch_ctx *, int64_t command_index);
/* gradient of the loss w.r.t. saved BN statistics is internal; the per-channel batch mean
 * and 1/sqrt(var+eps) of BN node `node` (C floats each) can be read back for tests. */
pooch_status pooch_get_bn_stats(pooch_ctx *, int32_t node, float *mean, float *istd);
/* Running averages of a BN layer's batch statistics, the quantities a trained network normalises with at
 * inference time (part of the training loop of section 2.1, though no step's loss or gradient depends on
 * them): every forward execution of the layer -- in pooch_step, and in the profiling passes, which are real
 * iterations (section 4.2) -- replaces
 *     mean <- decay * mean + (1 - decay) * batch mean
 *     var  <- decay * var  + (1 - decay) * batch variance * m / max(m - 1, 1)      (m = values per channel)
 * A re-forward (recompute class) normalises with the statistics saved by the forward pass and leaves the
 * averages alone, so they do not depend on the plan.  They start at mean 0, variance 1 when the graph is
 * finalized; decay defaults to 0.9 and may be changed at any time (1 freezes the averages, 0 keeps the last
 * batch's statistics).  get / set copy C floats each between host buffers and the context (a NULL pointer
 * skips that half); both synchronise.  POOCH_E_INVALID: not a BN layer, or decay outside [0, 1]. */
pooch_status pooch_set_bn_decay(pooch_ctx *, float decay);
pooch_status pooch_get_bn_running(pooch_ctx *, int32_t node, float *mean, float *var);
pooch_status pooch_set_bn_running(pooch_ctx *, int32_t node, const float *mean, const float *var);

/* ---- feature maps: the units being classified (section 4.1.1) --------------------------*/
int32_t pooch_num_nodes(pooch_ctx *);
int32_t pooch_num_fmaps(pooch_ctx *);
/* bytes = size inside the arena (256-byte rounded); producer = node id */
pooch_status pooch_fmap_info(pooch_ctx *, int32_t i, size_t *bytes, int32_t *producer);
/* bytes of the resident region (parameters, gradients, statistics, workspaces, input) */
size_t pooch_resident_bytes(pooch_ctx *);

/* ---- phase 1: runtime profiling (section 4.2) -------------------------------------------
 * Runs `warmup` untimed and `iters` timed steps with every map classified swap, timing each
 * layer's forward, backward and re-forward (the forward as a recomputation would run it)
 * and each map's swap-out / swap-in with HIP events; keeps the per-item median, in ms.
 * Array lengths: t_fwd, t_bwd, t_refwd -> num_nodes; t_out, t_in -> num_fmaps.
 * set_profile injects a profile (tests, CPU-only planning). */
pooch_status pooch_profile(pooch_ctx *, int warmup, int iters);
/* The same, one iteration at a time, for callers whose first training iterations double as the
 * profiling phase (section 4.1.2 places the profiling in the first few training iterations): each call
 * runs one all-swap step (forward + backward, gradients valid afterwards); timed != 0 adds its
 * durations to the samples.  pooch_finish_profile turns the samples into the profile (median). */
pooch_status pooch_profile_step(pooch_ctx *, int timed, float *loss_out);
pooch_status pooch_finish_profile(pooch_ctx *);
pooch_status pooch_get_profile(pooch_ctx *, double *t_fwd, double *t_bwd, double *t_refwd, double *t_out, double *t_in);
pooch_status pooch_set_profile(pooch_ctx *, const double *t_fwd, const double *t_bwd, const double *t_refwd,
                               const double *t_out, const double *t_in);
/* Beyond the paper: a second look at the durations.  The profiling pass above times every layer while
 * every map is being copied out and in (section 4.2), which slows the layers; a plan that copies little
 * then runs faster than simulated, and was chosen from pessimistic numbers.  pooch_refine_profile runs
 * `iters` >= 1 steps under the installed plan (ordinary iterations: loss and gradients are valid
 * afterwards) and replaces the forward, backward and re-forward durations of the layers that ran by
 * their medians in those steps; copy durations stay.  Call pooch_plan again afterwards.
 * POOCH_E_STATE without an installed plan, POOCH_E_NOPROFILE without a profile. */
pooch_status pooch_refine_profile(pooch_ctx *, int iters, float *loss_out);

/* ---- phase 2: classification (section 4.4) -----------------------------------------------
 * pooch_plan searches a classification for `mode` by simulating the step's timeline and
 * memory for each candidate (section 4.1.2) and installs the best one; predicted_ms (may be
 * NULL) receives its simulated step time.  max_bruteforce_bits caps the exponential part
 * of the keep/swap search (the binary tree over the maps whose swap-in is not hidden);
 * <= 0 selects the default.  POOCH_E_BUDGET when not even the all-swap plan fits.
 * pooch_set_plan installs an explicit classification (num_fmaps bytes, POOCH_KEEP/SWAP/
 * RECOMPUTE) after validating it the same way; `sched` != 0 enables moved-up swap-ins. */
pooch_status pooch_plan(pooch_ctx *, int mode, int max_bruteforce_bits, double *predicted_ms);
/* number of perturbed restarts of POOCH_MODE_REFINE's local search (default 8; deterministic: the
 * perturbations come from a fixed-seed generator) */
pooch_status pooch_set_search_effort(pooch_ctx *, int restarts);
pooch_status pooch_get_plan(pooch_ctx *, uint8_t *cls);
pooch_status pooch_set_plan(pooch_ctx *, const uint8_t *cls, int sched);
/* simulate without installing: step time (ms) and peak bytes of the dynamic region for an
 * explicit classification; POOCH_E_BUDGET if it does not fit. */
pooch_status pooch_simulate(pooch_ctx *, const uint8_t *cls, int sched, double *step_ms, size_t *peak_bytes);
/* number of timeline simulations the last pooch_plan ran (the paper's search-space sizes) */
int64_t pooch_plan_evaluations(pooch_ctx *);
/* the sets found on the all-swap timeline (section 4.4.2): in_LO[i], in_LI[i] are 0/1 per map */
pooch_status pooch_get_overhead_sets(pooch_ctx *, uint8_t *in_LO, uint8_t *in_LI);

/* test aid: the installed plan's command list, one row of 8 int64 per command:
 * kind, id, a0..a5 with kind 0 forward, 1 re-forward, 2 backward (id = layer; forward rows:
 * out, in0, in1 offsets; backward rows: dy, saved-tensor offset, then (offset, mode) of each
 * input's gradient, mode 0 none / 1 write / 2 accumulate / 3 reuse dy's buffer), 3 swap-out,
 * 4 swap-in (id = tensor; device offset, pinned offset), 5 record, 6 wait (id = stream 0
 * compute / 1 device-to-host / 2 host-to-device; a0 = event).  Offsets are relative to the
 * dynamic region (arena + resident bytes); -1 = none, -2 = the resident network input.
 * *nrows receives the number of commands; rows may be NULL to query it. */
pooch_status pooch_get_commands(pooch_ctx *, int64_t *rows, int64_t max_rows, int64_t *nrows);

/* ---- phase 3: execution -------------------------------------------------------------------
 * One forward + backward under the installed plan.  Enqueues everything, then synchronises
 * all three streams before returning; *loss_out (may be NULL) receives the mean loss. */
pooch_status pooch_step(pooch_ctx *, float *loss_out);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): pooch_step with the kernels' scratch -- the filter gradients' split-K partial sums, the batch
 * normalisations' reduction partials and per-tile statistics, the per-sample losses -- taken from an array that is
 * part of the library's code object (128 MiB = 134 217 728 bytes, held by every GPU the library runs on until the
 * process ends) instead of from the arena's resident region.  Same kernels, same command list, same bits as
 * pooch_step; inputs and outputs (arena, pinned buffer, streams, *loss_out) are the caller's as before.  The call
 * allocates nothing on the device or through the runtime: no hipMalloc / hipFree, no event creation (the plan's events
 * are made when the plan is installed), no torch call.
 * POOCH_E_BUDGET, with both sizes in pooch_last_error(), when the network's scratch exceeds the array (ResNet-50
 * needs 96 MiB at batch 640 and passes, 163 MiB at batch 2048 and does not; pooch_stats.scratch_bytes tells) -- checked first, so a planning-only context can ask;
 * POOCH_E_STATE without arena or plan; POOCH_E_HIP if the array's address could not be obtained when the context
 * was created.  All contexts on one GPU share that GPU's one array, which keeps the previous call's contents:
 * nothing in it has to start at zero (every range is written by the step before it is read), but two such calls
 * that overlap in time on one GPU -- from two contexts, or two threads -- race; serialise them. */
pooch_status pooch_step_static_scratch(pooch_ctx *, float *loss_out);

typedef struct pooch_stats {
    double step_ms;            /* wall time of the last step (host clock, enqueue to sync) */
    double predicted_ms;       /* simulated step time of the installed plan (0 without profile) */
    uint64_t swap_out_bytes;   /* bytes copied device -> host per step under the plan */
    uint64_t swap_in_bytes;    /* bytes copied host -> device per step */
    uint64_t peak_bytes;       /* high-water mark of the dynamic region (allocated bytes) */
    uint64_t extent_bytes;     /* highest arena offset ever touched + 1 minus lowest, dynamic region */
    uint64_t resident_bytes;
    uint64_t arena_bytes;
    int32_t n_keep, n_swap, n_recompute;
    int32_t n_commands;        /* length of the replayed command list */
    int32_t n_refwd;           /* forward re-executions per step */
    int32_t reserved;
    uint64_t scratch_bytes;    /* device scratch the kernels of a step use beyond their inputs and outputs (part of
                                  resident_bytes; what pooch_step_static_scratch needs of its static array) */
} pooch_stats;
pooch_status pooch_get_stats(pooch_ctx *, pooch_stats *);

/* Times one step with HIP events around every command and returns per-node milliseconds of
 * the installed plan's forward, backward and re-forward work (arrays of num_nodes doubles,
 * any may be NULL) -- the source of per-kernel rates in the benchmark.  ms_bwd_filter is the
 * part of a conv / fc layer's backward spent on the filter gradient (the data gradient takes
 * the rest of ms_bwd); zero for other layers. */
pooch_status pooch_step_timed(pooch_ctx *, float *loss_out, double *ms_fwd, double *ms_bwd, double *ms_refwd,
                              double *ms_bwd_filter);
/* name of the GPU kernel variant a conv / fc layer launches for part 0 forward, 1 data
 * gradient, 2 filter gradient, 3 forward when the layer is recomputed in backward (no
 * statistics for a following bn then) (static string, "" for other layers): lets a benchmark group
 * per-layer times by kernel, as a profiler's per-kernel summary does. */
const char *pooch_node_kernel(pooch_ctx *, int32_t node, int part);

/* measured pinned-copy rate of the host link: copies `bytes` each way `iters` times through
 * the context's copy streams and pinned buffer; GB/s (1e9) each way. */
pooch_status pooch_measure_link(pooch_ctx *, size_t bytes, int iters, double *d2h_gbs, double *h2d_gbs);

#ifdef __cplusplus
}
#endif
#endif /* POOCH_H */
