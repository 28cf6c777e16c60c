/*
 * vdnn.h - C ABI of the MI355X-native vDNN library (arxiv 1602.08124).
 *
 * The library runs the layer-wise CNN training step (Section 2.2 of the paper) with hand-written
 * HIP kernels for gfx950 and manages GPU memory the way Section 3 describes: layer-wise allocation
 * from a pool of fixed size, offload of a layer's input feature map X to pinned host memory during
 * forward propagation, prefetch during backward propagation, release as soon as data is dead,
 * under one of the transfer policies of Section 3.3.
 *
 * Conventions
 *   - every entry point returns a vdnn_status_t and never throws or aborts across the ABI;
 *     output parameters are untouched on error; vdnn_last_error() gives a message.
 *   - tensors are fp32, NCHW, dense.  Pointers are marked (host) or (device) below.
 *   - the caller owns descriptors and host arrays (consumed before the call returns); the library
 *     owns the net, its pinned host arena and its events.  The device pool and the two streams are
 *     borrowed from the caller when vdnn_attach_device() is used, otherwise created by the library
 *     (a third stream, on which fetches run, is always the library's own: one per process).
 *   - a net is not thread safe; calls on one net must be serialised by the caller.
 *   - all sizes are bytes unless a name says "count" (elements).
 */
#ifndef VDNN_H
#define VDNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vdnn_net vdnn_net_t; /* opaque, library-owned */

typedef enum {
    VDNN_OK = 0,
    VDNN_ERR_INVALID_ARG = 1,
    VDNN_ERR_OOM_DEVICE = 2, /* the step does not fit the GPU byte budget: the paper's "fails to train" */
    VDNN_ERR_OOM_HOST = 3,   /* pinned host arena could not be allocated */
    VDNN_ERR_HIP = 4,        /* a HIP runtime call failed */
    VDNN_ERR_STATE = 5,      /* call sequence error, e.g. backward without forward */
    VDNN_ERR_UNSUPPORTED = 6
} vdnn_status_t;

/* Section 3.3: static policies all / conv, the dynamic policy, and no offloading at all. */
typedef enum {
    VDNN_POLICY_NONE = 0, VDNN_POLICY_ALL = 1, VDNN_POLICY_CONV = 2, VDNN_POLICY_DYN = 3, /* Section 3.3 */
    VDNN_POLICY_FIT = 4,    /* not in the paper: see vdnn_set_policy */
    VDNN_POLICY_CUSTOM = 5  /* reported after vdnn_set_offload_set; not accepted by vdnn_set_policy */
} vdnn_policy_t;

/* Section 2.2 / 3.3: per CONV layer, the performance-optimal algorithm (needs workspace) or the
 * memory-optimal one (none).  GREEDY is what phase 3 of vDNN_dyn produces: performance-optimal except
 * where its workspace would overflow the budget. */
typedef enum { VDNN_ALGO_PERF = 0, VDNN_ALGO_MEM = 1, VDNN_ALGO_GREEDY = 2 } vdnn_conv_algo_t;
/* The kernels behind those algorithms.  Every pass of a CONV layer (forward, backward-data, backward-filter) can run
 *   GATHER    implicit GEMM that gathers X, dY and W as stored: no workspace, any shape (the memory-optimal algorithm);
 *   PACKED    implicit GEMM on a packed copy of W, with a deterministic split of long or ragged reductions: workspace
 *             of about |W| (backward-filter: one |W| per split); needs reduction channels in multiples of 16 (32 for
 *             backward-filter), an unstrided backward-data pass and tensors below 4 GiB;
 *   WINOGRAD  F(2x2,3x3) minimal filtering on wide 3x3 / stride 1 / pad 1 layers (256 reduction channels or more): 2.25x
 *             fewer multiplications, a workspace of hundreds of MiB (transformed filter, transformed tensors of a chunk
 *             of images, together within the chunk size of vdnn_op_set_winograd_chunk_bytes unless one image passes it);
 *   WINOGRAD_SMALL  the same on chunks of half as many images: a few per cent slower, about half the workspace (exists
 *             where a chunk of WINOGRAD holds two images or more).  Forward and backward-data results are the same
 *             bits as WINOGRAD's (the chunks partition the images); backward-filter sums over the chunks and differs in rounding.
 *   WINOGRAD4, WINOGRAD4_SMALL  F(4x4,3x3): 4x fewer multiplications and transformed tensors of 2.25x instead of 4x the
 *             tensor's size, from 128 reduction channels on; the fastest kernel where it applies (VGG-16 c3_2 forward at
 *             batch 256: 3.2 ms against 5.0 ms for F(2x2) and 6.7 ms for PACKED).  Its transforms carry factors up to 8
 *             and sixths: results lie about ten times further from the exact ones than F(2x2)'s, some 1e-5 of a tensor's
 *             largest value (inside the 1e-4 this library is tested to).
 * A net keeps, per CONV layer and direction, the list of ways it can run ordered by cost: WINOGRAD4, WINOGRAD4_SMALL,
 * WINOGRAD, WINOGRAD_SMALL, PACKED, GATHER until vdnn_profile has measured them on the GPU, by measured time afterwards.  The first entry is the layer's
 * performance-optimal algorithm, the last the memory-optimal one.  EVERY plan of the net (whatever the policy and the
 * budget) takes the first entry under VDNN_ALGO_PERF and fails with VDNN_ERR_OOM_DEVICE where that workspace does not
 * fit, so that plans under different policies and budgets compute the same bits; only VDNN_ALGO_GREEDY moves a layer
 * down its list (first entry whose workspace fits at that point of the step), and results then differ in rounding.
 * vdnn_set_winograd(net, 0) takes the four Winograd kernels off every list of the net, (net, 2) the two F(4x4) ones. */
typedef enum {
    VDNN_KERNEL_AUTO = -1, VDNN_KERNEL_GATHER = 0, VDNN_KERNEL_PACKED = 1, VDNN_KERNEL_WINOGRAD = 2, VDNN_KERNEL_WINOGRAD_SMALL = 3,
    VDNN_KERNEL_WINOGRAD4 = 4, VDNN_KERNEL_WINOGRAD4_SMALL = 5
} vdnn_conv_kernel_t;
typedef enum { VDNN_PASS_FWD = 0, VDNN_PASS_BWD_DATA = 1, VDNN_PASS_BWD_FILTER = 2 } vdnn_conv_pass_t;
#define VDNN_NO_KERNEL ((size_t)-1) /* vdnn_op_conv_workspace: the kernel does not apply to the shape */

typedef enum {
    VDNN_CONV = 0,       /* cross-correlation, zero padding, no bias */
    VDNN_RELU = 1,       /* in place: shares its input's feature map and gradient map */
    VDNN_MAXPOOL = 2,
    VDNN_AVGPOOL = 3,    /* divisor kernel*kernel, padded cells count as zeros */
    VDNN_FC = 4,         /* on the flattened NCHW vector, weight [out][in] */
    VDNN_CONCAT = 5,     /* along channels, in input order */
    VDNN_SOFTMAX_CE = 6  /* mean softmax cross-entropy over the batch; must be the last layer */
} vdnn_layer_type_t;

#define VDNN_MAX_INPUTS 8

typedef struct {
    int32_t type;                    /* vdnn_layer_type_t */
    int32_t n_inputs;                /* 1, except CONCAT (2..VDNN_MAX_INPUTS) */
    int32_t inputs[VDNN_MAX_INPUTS]; /* producer layer ids (< own id), -1 = the network input */
    int32_t out_channels;            /* CONV: output channels, FC: output features */
    int32_t kernel, stride, pad;     /* CONV and pools: square window */
} vdnn_layer_desc_t;

typedef struct {
    int32_t batch, in_c, in_h, in_w;
    int32_t n_layers;
    const vdnn_layer_desc_t* layers; /* (host) */
} vdnn_net_desc_t;

typedef struct {
    uint64_t budget_bytes;        /* 0 = unlimited */
    uint64_t cur_bytes;           /* live pool bytes now (after a step: W, dW, labels, loss) */
    uint64_t peak_bytes;          /* largest live total during the last planned step */
    uint64_t pool_extent_bytes;   /* address range the placement of that step needs (>= peak_bytes) */
    uint64_t baseline_bytes;      /* network-wide allocation of the baseline (Fig. 2 of the paper) */
    uint64_t persistent_bytes;    /* W + dW + labels + loss */
    double avg_bytes_layerstep;   /* mean of live bytes sampled at the start of every layer's fwd and bwd */
    uint64_t offloaded_bytes, prefetched_bytes; /* per step, device->host and host->device */
    uint64_t pinned_host_bytes;
    uint64_t workspace_bytes;     /* largest transient workspace of the step */
    int32_t n_offload, n_prefetch, n_ondemand_fetch; /* copies per step (a block that moves in pieces: one per piece) */
    int32_t effective_policy;     /* what DYN resolved to; otherwise the policy set */
    int32_t conv_algo;            /* vdnn_conv_algo_t of the current plan */
    int32_t n_memopt_convs;       /* CONV layers running the memory-optimal algorithm in fwd or bwd */
    int32_t window_fill_pm;       /* FIT / explicit set: share of the budget (per mille) the forward transfer windows fill; 0 = static schedule */
    int32_t window_fill_bwd_pm;   /* > 0: backward fetches are issued early, while live bytes stay within that share */
    int32_t n_winograd_convs;     /* CONV layers that run the Winograd kernel in any pass */
    int32_t n_downgraded_convs;   /* CONV layers that VDNN_ALGO_GREEDY moved off their performance-optimal entry in fwd or bwd */
    /* measured on the last executed step (0 until one has run) */
    double fwd_ms, bwd_ms, stall_ms, d2h_ms, h2d_ms, d2h_gbps, h2d_gbps;
} vdnn_mem_stats_t;

/* ---- the five calls of the paper's problem statement -------------------------------------- */

/* Builds the layer list, the dataflow graph with its consumer counts (Fig. nonlinear_dfg) and
 * the memory plan for policy NONE.  gpu_mem_budget covers everything on the device: feature
 * maps, gradient maps, W, dW, workspace (Section 3.2, "Memory Allocation/Release": one pool).
 * 0 means unlimited.  Host-only: does not touch the GPU. */
vdnn_status_t vdnn_create(const vdnn_net_desc_t* desc /*host*/, size_t gpu_mem_budget, vdnn_net_t** out);

/* Section 3.3.  ALL: offload the X of every CONV and POOL layer; CONV: only X that feed a CONV
 * layer; DYN: the profiling-pass sequence with out-of-memory as the signal:
 *   1. all with the memory-optimal algorithm must fit (else VDNN_ERR_OOM_DEVICE);
 *   2. performance-optimal algorithms with none, then conv, then all: adopt the first that fits;
 *   3. greedy: conv, then all, with each CONV layer moved down its list of kernels (vdnn_conv_kernel_t; the
 *      last entry is the memory-optimal algorithm) where its workspace would overflow the budget; else fall back to 1.
 * That order stands in for "fastest first".  After vdnn_profile (the paper's profiling passes, timed on the GPU) the
 * configurations of 2 and 3, and no offloading with the greedy downgrade, are all planned, and the one whose estimated
 * step (vdnn_estimate_step_ms) is shortest is adopted.
 * Static policies use the algorithm set by vdnn_set_conv_algo (default performance-optimal).
 * Re-plans the step.  Returns VDNN_ERR_OOM_DEVICE if the policy cannot fit the budget (the net
 * stays usable with its previous plan). */
vdnn_status_t vdnn_set_policy(vdnn_net_t*, vdnn_policy_t);
/* Which Winograd kernels the CONV layers of this net may run: 1 (default) all of them; 2 only the F(2x2,3x3) forms, whose
 * rounding error is a tenth of F(4x4,3x3)'s (for callers that want results within a few 1e-6 of the exact ones; VGG-16
 * at batch 256 then takes 146 instead of 114 ms per step); 0 none (direct kernels only: 186 ms).  Any other value:
 * VDNN_ERR_INVALID_ARG.  Takes effect at the next vdnn_set_policy / vdnn_set_offload_set. */
vdnn_status_t vdnn_set_winograd(vdnn_net_t*, int32_t enabled);
/* The list described above, as workspace bytes: entry 0 is what VDNN_ALGO_PERF allocates for the layer's forward
 * (bwd = 0) or backward (bwd != 0: the larger of backward-data and backward-filter) computation, the following entries
 * are what VDNN_ALGO_GREEDY falls back to, in order.  CONV: at least one entry, the last is 0.  FC: one entry (its
 * reduction-split partial sums).  Other layers: none.  count receives the number of entries, at most cap are written. */
vdnn_status_t vdnn_layer_workspace_options(const vdnn_net_t*, int layer, int32_t bwd, uint64_t* bytes /*host, may be NULL*/, size_t cap,
                                           size_t* count);
/* Names the kernels of a CONV layer (forward, backward-data, backward-filter): they become the layer's only way to run, in
 * every mode.  kernels = NULL gives the layer its list back.  VDNN_ERR_INVALID_ARG for a kernel that does not apply to the
 * layer's shape.  Takes effect at the next vdnn_set_policy / vdnn_set_offload_set.  With the kernels of a greedy plan named
 * on another net of the same shape, the two compute the same bits whatever their policies and budgets. */
vdnn_status_t vdnn_set_layer_kernels(vdnn_net_t*, int layer, const int32_t kernels[3] /*host, may be NULL*/);
/* The kernels (vdnn_conv_kernel_t) the current plan runs for a CONV layer's forward, backward-data and backward-filter pass. */
vdnn_status_t vdnn_layer_kernels(const vdnn_net_t*, int layer, int32_t kernels[3] /*host*/);
/* VDNN_POLICY_FIT goes beyond the paper.  Section 3.3 motivates vDNN_dyn by the cost of offloading more
 * than the budget asks for, and Section 3.1 by the distance between the two uses of X that a transfer can
 * hide behind; where arithmetic is fast relative to the host link, step time is simply bytes moved over
 * link rate.  FIT therefore
 *   (a) picks single feature maps (candidates: what ALL would offload): starting from none, while the step
 *       does not fit, it adds the smallest candidate whose addition makes it fit, else the largest remaining
 *       one; performance-optimal algorithms first, then the greedy downgrade, then memory-optimal;
 *   (b) keeps the paper's transfers (offload with the last forward consumer, fetches in findPrefetchLayer
 *       order) but not its end-of-layer synchronisation:
 *       forward: an offloaded X is released only when a later allocation would otherwise pass a share of the
 *       budget (oldest copy first); copies still on their way at the end of forward propagation are released in
 *       backward propagation, when an allocation needs the room or before the same feature map's fetch.
 *       While X is away its address range is lent out: a feature map that is not
 *       offloaded itself and had to release something becomes a tenant of the block released last, lined up
 *       from the low end of that range;
 *       backward: the fetch of X returns to the range X had (once its tenants are gone), and every fetch is
 *       issued as early as its own address range is free in the placement of the blocks (which, where the budget
 *       allows, keeps that range clear from the point at which live bytes alone would admit the fetch); the compute
 *       stream waits for a fetch just before the first computation that reads it.
 *       The forward share is the largest of 100, 99, ... 90, 88, ... 80, 75, 70, 60, 50, 0 % for which the
 *       blocks can be placed inside the budget (window_fill_pm in the stats; window_fill_bwd_pm = 1000 when
 *       fetches are issued early).
 *   (c) after vdnn_profile: improves the set of (a) by a local search on the estimated step time (drop a member,
 *       exchange one for one or two others, add one), does the same under the greedy kernel mode, and keeps the plan
 *       with the shortest estimate.
 * Values computed are bit-identical to every other policy as long as the plan's mode is performance-optimal (all such
 * plans of a net run the same kernels, see vdnn_conv_kernel_t; conv_algo in the stats tells).
 *
 * vdnn_set_offload_set: the same machinery with the set given by the caller.  buffers: (host) ids of feature
 * maps: -1 = the network input, otherwise the id of the layer that produces it (in-place ReLUs share their
 * input's id); each must be one that ALL would offload or the input of an FC layer (the paper manages the feature
 * extraction layers only and notes, at the start of Section 3, that the classification layers could be treated alike
 * for a smaller saving), else VDNN_ERR_INVALID_ARG.  window_fill_pm,
 * window_fill_bwd_pm (forward, backward): 0 = the paper's synchronisation, 1..1000 = transfer windows; forward
 * releases are postponed while live bytes stay within that share of the budget, backward fetches are issued
 * early while live bytes stay within that share of the budget and the address range is free.  Uses the
 * algorithm set by vdnn_set_conv_algo.  VDNN_ERR_OOM_DEVICE if it does not fit (previous plan kept).
 * vdnn_get_offload_set: the feature maps the current plan offloads (ascending); count receives how many,
 * at most cap are written.
 *
 * With transfer windows, a block larger than the part size (default 128 MiB) is copied, released and fetched
 * in at most 32 equal pieces, each following rule (b) on its own, so that one long copy does not hold up
 * every allocation behind it.  vdnn_set_window_part changes the part size (0 = whole blocks only); it takes
 * effect at the next vdnn_set_policy / vdnn_set_offload_set.  In the statistics n_offload, n_prefetch and
 * n_ondemand_fetch count copies, so a block that moves in pieces counts once per piece. */
vdnn_status_t vdnn_set_offload_set(vdnn_net_t*, const int32_t* buffers /*host*/, size_t count, int32_t window_fill_pm,
                                   int32_t window_fill_bwd_pm);
vdnn_status_t vdnn_set_window_part(vdnn_net_t*, size_t part_bytes);
vdnn_status_t vdnn_get_offload_set(const vdnn_net_t*, int32_t* buffers /*host, may be NULL*/, size_t cap, size_t* count);
/* Algorithm for the static policies; takes effect at the next vdnn_set_policy. */
vdnn_status_t vdnn_set_conv_algo(vdnn_net_t*, vdnn_conv_algo_t);

/* Section 3.3, "Dynamic vDNN": the profiling passes.  Runs every layer alone on the GPU (zero-filled tensors laid out in the
 * pool of the current plan, which therefore has to be one that fits): its forward and backward computation as a planned step
 * launches them, and for CONV layers every kernel that applies, pass by pass, `repeats` times each after a warm-up launch
 * (a kernel whose warm-up launch alone takes more than 8 times the fastest kernel measured for the pass, and more than
 * 20 ms, is not repeated: that one time is its figure); and measures the rate of the host link in both directions.  Afterwards each CONV layer's list (vdnn_conv_kernel_t) is
 * ordered by measured time, and vdnn_set_policy(DYN) / (FIT) choose by estimated step time (see there).  Overwrites dW and
 * whatever the pool holds above the weights; weights stay.  Takes effect at the next vdnn_set_policy / vdnn_set_offload_set.
 * vdnn_set_layer_profile / vdnn_set_link_rate put numbers in by hand (a profile kept from an earlier run; tests of the
 * host logic, which need no GPU): pass is a vdnn_conv_pass_t for CONV layers, 0 = forward / 1 = backward (kernel ignored)
 * for all others; ms >= 0.  vdnn_get_layer_profile: ms < 0 = not measured. */
vdnn_status_t vdnn_profile(vdnn_net_t*, int32_t repeats);
vdnn_status_t vdnn_set_layer_profile(vdnn_net_t*, int layer, int32_t pass, int32_t kernel, float ms);
vdnn_status_t vdnn_get_layer_profile(const vdnn_net_t*, int layer, int32_t pass, int32_t kernel, float* ms /*host*/);
/* Duration of the current plan's step as the profile predicts it: the op list replayed on two timelines (Section 3.2: the
 * compute stream and the memory stream), a layer taking its measured time, a copy its bytes over the measured link rate,
 * the two meeting where the plan synchronises them.  VDNN_ERR_STATE without a profile or a valid plan. */
vdnn_status_t vdnn_estimate_step_ms(const vdnn_net_t*, double* ms /*host*/);
vdnn_status_t vdnn_set_link_rate(vdnn_net_t*, double d2h_gbps, double h2d_gbps);
vdnn_status_t vdnn_get_link_rate(const vdnn_net_t*, double* d2h_gbps /*host*/, double* h2d_gbps /*host*/);

/* Forward propagation, layers 0..L-1 (Section 2.2; offload per Section 3.2 "Memory Offload").
 * input: (device) batch*in_c*in_h*in_w floats; labels: (device) batch int32 in [0, classes).
 * Both are copied into the pool before use.  loss_out: (host) mean softmax-CE loss.
 * Returns once the forward computations have completed on the GPU and the loss has been read.  Under the schedules with
 * transfer windows (VDNN_POLICY_FIT, vdnn_set_offload_set with a fill) offload copies may still be on their way then: they
 * go on beside the first backward computations, and their device blocks are released there (Section 3.2 ends every
 * offload with its layer; the paper's own policies do exactly that).  vdnn_get_output waits for the copy it reads.
 * A label outside [0, classes) is never used as an index: the call then returns VDNN_ERR_INVALID_ARG after the pass
 * (loss_out untouched, no backward pass possible). */
vdnn_status_t vdnn_forward(vdnn_net_t*, const float* input, const int32_t* labels, float* loss_out);

/* Backward propagation, layers L-1..0 (Eq. chain_rule; prefetch per Section 3.2 "Memory Prefetch").
 * Leaves every dW in the pool.  Returns after completion on the GPU: computations, offload copies that forward
 * propagation left in flight, and fetches.  Offloads run on the memory stream, fetches on a stream the library owns
 * (one per process, default priority), so that a fetch never queues behind an offload.  The transfer and stall figures of
 * vdnn_mem_stats (d2h_ms, h2d_ms, d2h_gbps, h2d_gbps, stall_ms) are those of the whole step and final after this call. */
vdnn_status_t vdnn_backward(vdnn_net_t*);

/* Figures 11/12 of the paper: maximum and average memory, offloaded bytes; plus measured times. */
vdnn_status_t vdnn_mem_stats(const vdnn_net_t*, vdnn_mem_stats_t* out /*host*/);

/* ---- what the five need in order to be usable and testable ------------------------------- */

/* Borrow device memory and streams (e.g. torch-owned).  pool_bytes must be >= pool_extent_bytes
 * of the current plan.  stream_* are hipStream_t.  Without this call the library allocates its
 * own pool (hipMalloc) and streams on first use. */
vdnn_status_t vdnn_attach_device(vdnn_net_t*, void* pool_base /*device*/, size_t pool_bytes, void* stream_compute,
                                 void* stream_memory);

/* Weights: CONV [K][C][R][S], FC [out][in], fp32 (host).  count must match. */
vdnn_status_t vdnn_set_weights(vdnn_net_t*, int layer, const float* w /*host*/, size_t count);
vdnn_status_t vdnn_get_weight_grad(vdnn_net_t*, int layer, float* dw /*host*/, size_t count);
vdnn_status_t vdnn_get_weights(vdnn_net_t*, int layer, float* w /*host*/, size_t count);
size_t vdnn_weight_count(const vdnn_net_t*, int layer); /* 0 for layers without weights */
/* Section 2.2: once backward propagation reaches the first layer the weights are adjusted with the
 * weight gradients.  Plain SGD on every layer: W <- W - learning_rate * dW.  Call after vdnn_backward. */
vdnn_status_t vdnn_sgd_step(vdnn_net_t*, float learning_rate);
size_t vdnn_output_count(const vdnn_net_t*, int layer); /* elements of the layer's output */

/* Copies a layer's output as it stands at the end of forward propagation (layer = -1: the logits, i.e. the input of the
 * loss layer); valid between a completed vdnn_forward and the vdnn_backward that follows.  An in-place ReLU shares its
 * producer's feature map, so for both layers this is the value after the ReLU.  The copy comes from the pool, or from the
 * pinned host arena when the current plan has offloaded that feature map.  VDNN_ERR_STATE when the feature map was released
 * during forward propagation because no backward computation reads it (use vdnn_capture_output for those). */
vdnn_status_t vdnn_get_output(vdnn_net_t*, int layer, float* dst /*host*/, size_t count);

/* Test hooks: copy layer's output Y (right after its forward computation) / the gradient w.r.t.
 * its output dY (right before its backward computation) to a host array during the next
 * passes.  dst = NULL removes the hook.  The copies synchronise the compute stream. */
vdnn_status_t vdnn_capture_output(vdnn_net_t*, int layer, float* dst /*host*/);
vdnn_status_t vdnn_capture_grad(vdnn_net_t*, int layer, float* dst /*host*/);

/* Per-layer times of the compute stream (Section 3.2's argument is per layer: a transfer hides behind a layer
 * whose computation takes longer than the copy).  With timing on, every pass records an event at the start of
 * each layer; a layer's time runs from its start to the start of the next layer of the pass (or the end of
 * the pass) and therefore includes any wait for a transfer.  vdnn_layer_times copies the times of the last
 * forward and backward pass (milliseconds; count = number of layers; VDNN_ERR_STATE before a timed step). */
vdnn_status_t vdnn_set_layer_timing(vdnn_net_t*, int32_t on);
vdnn_status_t vdnn_layer_times(const vdnn_net_t*, float* fwd_ms /*host*/, float* bwd_ms /*host*/, size_t count);

/* The planned step as text, one op per line: "<where> <op> <tag> <bytes> [<offset>]" with
 * where = create | F<layer> | B<layer>, op = alloc | free | offload | prefetch | ondemand | compute.
 * Writes at most cap bytes (NUL-terminated) and stores the full length in *needed. */
vdnn_status_t vdnn_trace(const vdnn_net_t*, char* buf /*host*/, size_t cap, size_t* needed);

const char* vdnn_last_error(const vdnn_net_t*);
void vdnn_destroy(vdnn_net_t*);

/* ---- single-layer entry points (the kernels behind the step; all pointers are device) ----- */
/* Message of the last failing vdnn_op_* call of this thread. */
const char* vdnn_op_last_error(void);
/* stream: hipStream_t or NULL.  Shapes: X [N][C][H][W], W [K][C][R][S], Y [N][K][P][Q] with
 * P = (H + 2 pad - R)/stride + 1.  Asynchronous on the stream.  A tensor may have at most 2^31 - 2 elements:
 * larger shapes return VDNN_ERR_INVALID_ARG before anything is launched (vdnn_create: VDNN_ERR_UNSUPPORTED). */

/* Convolution kernels in the sense of Section 2.2's memory-optimal / performance-optimal trade-off (vdnn_conv_kernel_t):
 *  - GATHER: no workspace, implicit GEMM whose gather works directly on W as stored (memory-optimal);
 *  - PACKED: one packed copy of W (+ partial sums of split tiles): the faster implicit-GEMM kernel; applies when the reduction
 *    channels are a multiple of 16, backward-data is unstrided and the tensors are below 4 GiB;
 *  - WINOGRAD F(2x2,3x3) on 3x3 / stride 1 / pad 1 layers, reduction channels a multiple of 16,
 *    at least 256 of them, output channels of the pass a multiple of 4 and at least 128 (backward-filter: input
 *    channels a multiple of 128, 256 or more output channels): transformed
 *    filter (16/9 of W) plus transformed input and products for a chunk of images (together at most the chunk size below);
 *  - WINOGRAD4 F(4x4,3x3) on the same layers and on those with 128 to 255 reduction channels (backward-filter: 128 or more
 *    output channels): transformed filter 36/9 = 4 times W, transformed tensors 2.25 times the tensor;
 *  - the _SMALL forms of both on chunks of half as many images.
 * vdnn_op_conv_workspace(pass, kernel, shape) returns the bytes that kernel needs (VDNN_NO_KERNEL: it does not apply);
 * vdnn_op_conv_*_workspace() the bytes of the fastest kernel that applies to the shape (0: only GATHER).
 * The three conv entry points take the kernel to run: an explicit one returns VDNN_ERR_INVALID_ARG where it does not
 * apply or workspace_bytes is too small for it (nothing is launched); VDNN_KERNEL_AUTO runs the fastest kernel the
 * given workspace has room for (NULL: GATHER).  Results
 * agree to rounding (F(2x2): a few 1e-6 of the largest output, F(4x4): about 1e-5); each kernel is deterministic. */
size_t vdnn_op_conv_workspace(int pass /*vdnn_conv_pass_t*/, int kernel /*vdnn_conv_kernel_t, not AUTO*/, int N, int C, int H, int W, int K,
                              int R, int S, int stride, int pad);
/* Process-wide chunk size of the Winograd workspaces in bytes (0 restores the default, 384 MiB): a workspace holds the
 * transformed filter (backward-filter: the products and their partial sums) and the transformed tensors of as many
 * images as fit beside it, at least one.  Workspace sizes and plans derive from it: set it before creating nets, not
 * while one exists. */
void vdnn_op_set_winograd_chunk_bytes(size_t bytes);
size_t vdnn_op_conv_fwd_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
size_t vdnn_op_conv_bwd_data_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
/* Y = conv(X, W); relu != 0 applies max(.,0) to the result in the same kernel. */
vdnn_status_t vdnn_op_conv_fwd(const float* x, const float* w, float* y, void* workspace, size_t workspace_bytes, int N, int C,
                               int H, int W, int K, int R, int S, int stride, int pad, int relu, int kernel, void* stream);
/* dX = sum over the forward terms that touched it (Eq. chain_rule).  relu_mask (may be NULL): a tensor of
 * dX's shape, the output of an in-place ReLU that produced X; dX is zeroed where it is not positive,
 * which is that ReLU's backward computation folded into this kernel's store. */
vdnn_status_t vdnn_op_conv_bwd_data(const float* dy, const float* w, float* dx, void* workspace, size_t workspace_bytes, int N,
                                    int C, int H, int W, int K, int R, int S, int stride, int pad, const float* relu_mask,
                                    int kernel, void* stream);
/* dW; the reduction over N*P*Q is split, partial sums go to workspace and are added in a fixed
 * order (deterministic, no atomics).  The workspace query returns the bytes of the fastest algorithm for the shape
 * (Winograd where the rule above admits it: the 16 accumulated products, their partial sums, and the transformed
 * X and dY of a chunk of images); with less the direct split kernel runs if its partial sums fit, and with workspace
 * NULL or too small for those the memory-optimal algorithm: no split, one workgroup per output tile (much slower on
 * long reductions). */
size_t vdnn_op_conv_bwd_filter_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
vdnn_status_t vdnn_op_conv_bwd_filter(const float* x, const float* dy, float* dw, void* workspace, size_t workspace_bytes,
                                      int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int kernel, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): vdnn_op_conv_bwd_filter with the workspace taken from a static device buffer of VDNN_STATIC_SCRATCH_BYTES
 * that the library holds on every GPU it runs on until the process ends.  The call allocates and frees nothing.  kernel as
 * above, except that VDNN_KERNEL_AUTO means the fastest kernel that applies to the shape (the one
 * vdnn_op_conv_bwd_filter_workspace sizes for).  A kernel whose workspace is larger than the buffer is refused with
 * VDNN_ERR_INVALID_ARG and a message (nothing is launched): pick a smaller kernel (GATHER needs none) or use the entry point
 * above.  Same kernels, same results bit for bit as vdnn_op_conv_bwd_filter given a workspace of that size.  All calls on one
 * GPU share the buffer: calls that overlap there (different streams, different threads) race; calls on one stream do not.
 * The first call on a GPU looks the buffer's address up (no allocation by this library; make it before a capture starts). */
#define VDNN_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
vdnn_status_t vdnn_op_conv_bwd_filter_static(const float* x, const float* dy, float* dw, int N, int C, int H, int W, int K, int R, int S,
                                             int stride, int pad, int kernel, void* stream);

/* FC: Y[N][O] = X[N][I] W[O][I]^T ; dX = dY W ; dW = dY^T X.  Same workspace rule (too little: no split). */
size_t vdnn_op_fc_workspace(int N, int I, int O, int which /*0 fwd, 1 bwd-data, 2 bwd-filter*/);
vdnn_status_t vdnn_op_fc_fwd(const float* x, const float* w, float* y, void* workspace, size_t workspace_bytes, int N, int I,
                             int O, void* stream);
vdnn_status_t vdnn_op_fc_bwd_data(const float* dy, const float* w, float* dx, void* workspace, size_t workspace_bytes, int N,
                                  int I, int O, void* stream);
vdnn_status_t vdnn_op_fc_bwd_filter(const float* x, const float* dy, float* dw, void* workspace, size_t workspace_bytes, int N,
                                    int I, int O, void* stream);

vdnn_status_t vdnn_op_relu_fwd(float* y, size_t count, void* stream);                  /* in place */
vdnn_status_t vdnn_op_relu_bwd(const float* y, float* dy, size_t count, void* stream); /* in place on dy, mask y > 0 */
vdnn_status_t vdnn_op_maxpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, void* stream);
/* first maximum in row-major window order takes the gradient; overlapping windows add up.
 * relu_mask != 0: X is the output of an in-place ReLU whose backward is folded in (dX = 0 where X <= 0). */
vdnn_status_t vdnn_op_maxpool_bwd(const float* x, const float* dy, float* dx, int N, int C, int H, int W, int k, int stride,
                                  int pad, int relu_mask, void* stream);
vdnn_status_t vdnn_op_avgpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, void* stream);
vdnn_status_t vdnn_op_avgpool_bwd(const float* dy, float* dx, int N, int C, int H, int W, int k, int stride, int pad, void* stream);
/* loss: (device) one float, mean over the batch.  dz = (softmax(z) - onehot)/N.  A label outside [0, classes) is never
 * used as an index: its row makes the loss NaN, and its dz has no onehot term. */
vdnn_status_t vdnn_op_softmax_ce_fwd(const float* z, const int32_t* labels, float* loss, int N, int classes, void* stream);
vdnn_status_t vdnn_op_softmax_ce_bwd(const float* z, const int32_t* labels, float* dz, int N, int classes, void* stream);
/* to_big != 0 (concat forward):  big[n][c_off + c][hw] = small[n][c][hw], src = small, dst = big.
 * to_big == 0 (concat backward): small[n][c][hw] = big[n][c_off + c][hw], src = big,   dst = small. */
vdnn_status_t vdnn_op_concat_copy(const float* src, float* dst, int N, int c_small, int c_big, int c_off, int hw, int to_big,
                                  void* stream);
vdnn_status_t vdnn_op_add(float* acc, const float* src, size_t count, void* stream); /* acc += src */

#ifdef __cplusplus
}
#endif
#endif /* VDNN_H */
