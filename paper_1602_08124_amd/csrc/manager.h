// Host-side vDNN memory manager: dataflow graph, transfer policy, step planner and executor.
//
// The training step of a fixed network is a fixed sequence of operations, so the manager compiles
// it once per (network, policy, budget) into a "plan": an ordered list of ops (allocate, release,
// offload, prefetch, compute ...) together with the byte offset of every block inside the pool.
// Executing a step replays the plan on two HIP streams.  Nothing on the step path calls
// hipMalloc/hipFree (Section 3.2, "Memory Allocation/Release").  Planning is pure host code and
// needs no GPU, which is also how vDNN_dyn tests trainability (Section 3.3).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <string>
#include <vector>

#include "../../include/vdnn.h"
#include "ops.h"

namespace vdnn {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t n) { return (n + kAlign - 1) / kAlign * kAlign; }

struct Layer {
    int type = 0;
    std::vector<int> inputs;
    int out = 0, k = 0, stride = 1, pad = 0;
    int C = 0, H = 0, W = 0;  // output shape (per image)
    int buf = 0;              // feature-map buffer holding the output (-1 = network input)
    size_t wcount = 0;        // weight elements
    // Kernel fusion of in-place ReLU layers (same values, fewer passes over HBM):
    int relu_after = -1;      // CONV: the ReLU living in its output whose forward runs in the conv's epilogue
    int relu_before = -1;     // CONV / MAXPOOL: the ReLU living in its input whose backward runs in this layer's dX store
    int fwd_folded_into = -1, bwd_folded_into = -1;  // RELU: the layer that does its work (or -1)
};

// A feature-map buffer: produced by one non-in-place layer (or the network input), possibly
// overwritten in place by activation layers, read by `readers`.
struct Buffer {
    size_t count = 0;          // elements
    int C = 0, H = 0, W = 0;
    std::vector<int> readers;  // non-in-place layers that read it, ascending
    std::vector<int> inplace;  // in-place layers living in it
    std::vector<int> bwd_users;  // layers whose backward computation reads its contents, ascending
};

enum OpKind {
    OP_SAMPLE,       // start of a layer's fwd/bwd: sample live bytes
    OP_ALLOC,
    OP_FREE,
    OP_LOAD_INPUT,   // copy the caller's batch and labels into the pool
    OP_OFFLOAD,      // issue device->host copy of a buffer on the memory stream
    OP_WAIT_COPY,    // compute stream waits for a copy issued earlier (end-of-layer synchronisation)
    OP_PREFETCH,     // issue host->device copy on the memory stream
    OP_ONDEMAND,     // host->device copy the compute stream waits for immediately
    OP_FWD,
    OP_BWD,
};

struct Op {
    OpKind kind;
    int phase;       // 0 create, 1 forward, 2 backward
    int layer;       // -1 for the input load
    int block = -1;  // ALLOC/FREE/OFFLOAD/PREFETCH/ONDEMAND: the block; WAIT_COPY: block whose copy is awaited
    int part = -1;   // the same ops on one piece of a block that moves in pieces (-1 = the whole block)
    int buf = -2;    // buffer id for transfers
    // compute ops
    std::vector<int> in_blocks;    // blocks holding the layer's inputs
    int out_block = -1;            // Y (fwd) / the buffer itself for in-place layers
    int gin_block = -1;            // dY
    std::vector<int> gout_blocks;  // dX per input (-1 = not needed); a temp block when accumulate is set
    std::vector<int> gacc_blocks;  // when >= 0: add gout_blocks[i] into this block afterwards
    int ws_block = -1;
    int kern[3] = {0, 0, 0};       // CONV: the kernel of forward / backward-data / backward-filter (ops.h)
};

// One way to run a CONV layer's forward computation (fwd) or its backward computation (bd + bf, which share one
// workspace block): the kernels, the workspace they need and what they cost (milliseconds once the layer has
// been profiled, a rank before).  Section 3.3: the profiled algorithms of a layer, fastest first.
struct KernelOption {
    int fwd = 0, bd = 0, bf = 0;
    size_t ws = 0;
    double cost = 0.0;
};

// Section 3.3, "Dynamic vDNN": what the profiling passes measure.  Times in milliseconds, < 0 = not measured.
struct LayerProfile {
    float conv[3][kNumKernels];                                      // CONV: [pass][kernel]; -1 = not measured
    LayerProfile() {
        for (auto& pass : conv)
            for (float& ms : pass) ms = -1.f;
    }
    float fwd = -1, bwd = -1;                                        // every layer: the kernels its plan entry runs
};

struct Block {
    std::string tag;
    size_t bytes = 0;  // aligned
    size_t raw = 0;
    int t0 = 0, t1 = 0;  // op indices [t0, t1)
    size_t offset = 0;
    bool persistent = false;
    size_t host_off = 0;  // offset in the pinned arena (buffers that are offloaded)
    int buf = -2;  // feature-map buffer the block holds (-1 = network input), -2 = something else
    // Range lending (transfer windows): while an offloaded block is away its address range takes in later
    // feature maps (tenants), and the fetch of the same buffer (twin) returns to it.  Tenants and twin are
    // placed together with the host, at fixed distances from its offset.
    int host = -1;        // block whose range this one lives in
    size_t host_rel = 0;  // byte distance from the host's offset
    // A block that is copied in pieces: `parts` pieces of part_bytes (the last one shorter), which share the
    // block's address range but are released (forward) or allocated (backward) one by one.
    int parts = 1;
    size_t part_bytes = 0;
    std::vector<int> part_t0, part_t1;  // lifetime of each piece, op indices [t0, t1)
    size_t piece_bytes(int i) const { return parts == 1 ? bytes : std::min(part_bytes, bytes - (size_t)i * part_bytes); }
    size_t piece_raw(int i) const {
        if (parts == 1) return raw;
        const size_t lo = (size_t)i * part_bytes;
        return raw > lo ? std::min(part_bytes, raw - lo) : 0;
    }
};

struct Plan {
    bool ok = false;
    std::string fail_where, fail_why;
    int policy = 0;
    std::vector<Op> ops;
    std::vector<Block> blocks;
    int first_fwd_op = 0, first_bwd_op = 0;
    size_t peak = 0, extent = 0, persistent = 0, pinned = 0, max_ws = 0;
    double avg = 0.0;
    size_t offloaded = 0, prefetched = 0;
    int n_offload = 0, n_prefetch = 0, n_ondemand = 0;
    int labels_block = -1, loss_block = -1;
    std::vector<int> w_block, dw_block;  // per layer: persistent blocks of W and dW (-1 for layers without weights)
    int algo = 0;                        // vdnn_conv_algo_t the plan was compiled with
    std::vector<char> memopt_fwd, memopt_bwd;  // per layer: the mode (memory-optimal, or a greedy downgrade) put the CONV layer on the no-workspace kernel
    std::vector<int> opt_fwd, opt_bwd;   // per CONV layer: index of the KernelOption the plan runs (-1 elsewhere)
    int n_memopt = 0;
    int n_downgraded = 0;                // CONV layers that the greedy mode moved off their performance-optimal option in fwd or bwd
    int n_winograd = 0;                  // CONV layers that run the Winograd kernel in any pass
    std::vector<char> offload_set;  // buffer id + 1 -> this step offloads it
    int fill_pm = 0, fill_bwd_pm = 0;  // share of the budget (per mille) the transfer windows may fill in forward / backward; 0 = static schedule
};

}  // namespace vdnn

struct vdnn_net {
    int batch = 0, in_c = 0, in_h = 0, in_w = 0;
    std::vector<vdnn::Layer> layers;
    std::vector<vdnn::Buffer> bufs;  // index = buffer id + 1
    size_t budget = 0;               // 0 = unlimited
    size_t part_bytes = (size_t)128 << 20;  // transfer windows move larger blocks in pieces of about this size (0 = whole blocks)
    int policy = VDNN_POLICY_NONE, effective = VDNN_POLICY_NONE;
    int static_algo = VDNN_ALGO_PERF;
    int winograd = 1;      // which Winograd kernels are among the options of 3x3 layers: 0 none, 1 all, 2 only F(2x2, 3x3)
    // Per layer, how it can run, preference order (first = performance-optimal, last of a CONV layer = memory-optimal, no
    // workspace).  Every plan of the net takes its kernels from here, so that plans under different policies and budgets
    // compute the same bits; only the greedy mode (Section 3.3, phase 3) moves a layer down its list.
    std::vector<std::vector<vdnn::KernelOption>> options_fwd, options_bwd;
    std::vector<int> pinned_kernels;  // per layer: -1, or fwd | bd << 4 | bf << 8 set by vdnn_set_layer_kernels (the layer's only option then)
    std::vector<vdnn::LayerProfile> profile;
    bool profiled = false;
    double link_d2h_gbps = 0.0, link_h2d_gbps = 0.0;  // measured by the profiling pass (0: not measured)
    vdnn::Plan plan;
    size_t baseline = 0;

    // device side
    char* pool = nullptr;
    size_t pool_bytes = 0;
    bool own_pool = false, weights_set = false;
    hipStream_t sc = nullptr, sm = nullptr;
    hipStream_t sf = nullptr;  // host->device fetches (the library's own; offloads use sm)
    bool have_streams = false, own_streams = false;
    char* pinned = nullptr;
    size_t pinned_bytes = 0;
    std::vector<hipEvent_t> events;
    int events_used = 0;

    bool fwd_done = false;
    std::vector<float*> cap_out, cap_grad;
    std::string err;

    // measured on the last step
    double fwd_ms = 0, bwd_ms = 0, stall_ms = 0, d2h_ms = 0, h2d_ms = 0;
    struct Timed { int e0, e1; size_t bytes; int dir; };
    std::vector<Timed> copies;
    struct Stall { int e_compute, e_copy; };
    std::vector<Stall> stalls;
    int ev_f0 = -1, ev_f1 = -1, ev_b0 = -1, ev_b1 = -1;
    bool time_layers = false;                    // record an event at the start of every layer's fwd / bwd
    std::vector<std::pair<int, int>> layer_marks;  // (layer, event) in execution order of the current pass
    std::vector<float> layer_fwd_ms, layer_bwd_ms;
    std::vector<int> copy_done_event;  // per block: event recorded after its last copy

    vdnn::Buffer& B(int id) { return bufs[id + 1]; }
    const vdnn::Buffer& B(int id) const { return bufs[id + 1]; }
};

// ---- shared by graph.cpp, planner.cpp and manager.cpp ----------------------------------------------------
namespace vdnn {

inline bool in_place(int type) { return type == VDNN_RELU; }
inline bool needs_x_in_bwd(int type) { return type == VDNN_CONV || type == VDNN_MAXPOOL || type == VDNN_FC || type == VDNN_SOFTMAX_CE; }
inline const char* type_name(int t) {
    static const char* n[] = {"conv", "relu", "maxpool", "avgpool", "fc", "concat", "softmax_ce"};
    return (t >= 0 && t <= 6) ? n[t] : "?";
}

inline std::string fmt(const char* f, ...) {
    char b[512];
    va_list ap;
    va_start(ap, f);
    vsnprintf(b, sizeof b, f, ap);
    va_end(ap);
    return b;
}

inline int buf_of(const vdnn_net& n, int layer) { return layer < 0 ? -1 : n.layers[layer].buf; }

inline void shape_of(const vdnn_net& n, int layer, int* C, int* H, int* W) {
    if (layer < 0) { *C = n.in_c; *H = n.in_h; *W = n.in_w; }
    else { *C = n.layers[layer].C; *H = n.layers[layer].H; *W = n.layers[layer].W; }
}

// graph.cpp
vdnn_status_t build_graph(vdnn_net& n, const vdnn_net_desc_t* d, std::string& err);
bool fold_fwd(const vdnn_net& n, int conv);     // the conv applies the ReLU living in its output
bool fold_bwd(const vdnn_net& n, int reader);   // the reader applies the backward of the ReLU living in its input
void build_kernel_options(vdnn_net& n);  // from shapes, n.winograd and, when there is one, the profile
bool selected(const vdnn_net& n, int b, int policy);
size_t baseline_bytes(const vdnn_net& n);

// planner.cpp
// offload_set (indexed by buffer id + 1), when given, replaces the policy's choice of feature maps; place = false
// stops after the byte accounting (p.ok then only says that the live total fits); fill_pm / fill_bwd_pm > 0 turn the
// transfer windows on.
void compile_plan(const vdnn_net& n, int policy, int algo, Plan& p, const std::vector<char>* offload_set = nullptr, bool place = true,
                  int fill_pm = 0, int fill_bwd_pm = 0, int place_rounds = 300);
vdnn_status_t plan_policy(vdnn_net& n, int policy);
double estimate_step_ms(const vdnn_net& n, const Plan& p);  // from the profile; < 0 without one

}  // namespace vdnn
