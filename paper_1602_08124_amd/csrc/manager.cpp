// vDNN memory manager, device side: pool and pinned arena, execution of a planned step on two HIP streams, timing,
// and the C ABI.  Graph construction lives in graph.cpp, planning in planner.cpp; see manager.h for the overall shape.
#include "manager.h"

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>

#include "ops.h"

using namespace vdnn;

// ---------------------------------------------------------------------------------------------
// device plumbing
// ---------------------------------------------------------------------------------------------
#define HIPCHK(call)                                                                             \
    do {                                                                                         \
        hipError_t e__ = (call);                                                                 \
        if (e__ != hipSuccess) {                                                                 \
            n.err = fmt("%s failed: %s (%s:%d)", #call, hipGetErrorString(e__), __FILE__, __LINE__); \
            return VDNN_ERR_HIP;                                                                 \
        }                                                                                        \
    } while (0)

// One stream for host->device fetches, shared by every net of the process (a process that keeps creating streams ends up
// with several of them on one hardware queue, where copies and kernels of different streams serialise).
static hipStream_t fetch_stream() {
    static hipStream_t st = nullptr;
    static std::once_flag once;
    std::call_once(once, []() {
        if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) { (void)hipGetLastError(); st = nullptr; }
    });
    return st;
}

static vdnn_status_t ensure_device(vdnn_net& n) {
    if (!n.plan.ok) { n.err = "no valid plan (the current policy does not fit the budget)"; return VDNN_ERR_STATE; }
    if (!n.sf) n.sf = fetch_stream();   // null: fetches share the memory stream
    if (!n.have_streams) {
        HIPCHK(hipStreamCreateWithFlags(&n.sc, hipStreamNonBlocking));
        HIPCHK(hipStreamCreateWithFlags(&n.sm, hipStreamNonBlocking));
        n.have_streams = n.own_streams = true;
    }
    if (!n.pool || n.pool_bytes < n.plan.extent) {
        if (n.pool && !n.own_pool) {
            n.err = fmt("attached pool of %zu bytes is smaller than the plan's extent %zu", n.pool_bytes, n.plan.extent);
            return VDNN_ERR_INVALID_ARG;
        }
        const size_t want = n.budget ? n.budget / kAlign * kAlign : n.plan.extent;
        char* fresh = nullptr;
        HIPCHK(hipMalloc((void**)&fresh, want));
        if (n.pool) {  // keep W (persistent region sits at the bottom of the pool)
            HIPCHK(hipMemcpy(fresh, n.pool, n.plan.persistent, hipMemcpyDeviceToDevice));
            HIPCHK(hipFree(n.pool));
        }
        n.pool = fresh; n.pool_bytes = want; n.own_pool = true;
    }
    if (n.plan.pinned > n.pinned_bytes) {
        if (n.pinned) { HIPCHK(hipHostFree(n.pinned)); n.pinned = nullptr; n.pinned_bytes = 0; }
        hipError_t e = hipHostMalloc((void**)&n.pinned, n.plan.pinned, hipHostMallocDefault);
        if (e != hipSuccess) {
            n.err = fmt("pinned host arena of %zu bytes: %s", n.plan.pinned, hipGetErrorString(e));
            (void)hipGetLastError();
            n.pinned = nullptr;
            return VDNN_ERR_OOM_HOST;
        }
        n.pinned_bytes = n.plan.pinned;
    }
    return VDNN_OK;
}

static int new_event(vdnn_net& n, hipError_t* err) {
    if (n.events_used == (int)n.events.size()) {
        hipEvent_t e;
        *err = hipEventCreate(&e);
        if (*err != hipSuccess) return -1;
        n.events.push_back(e);
    }
    *err = hipSuccess;
    return n.events_used++;
}

#define NEWEV(var)                                   \
    int var;                                         \
    {                                                \
        hipError_t ee__;                             \
        var = new_event(n, &ee__);                   \
        if (var < 0) HIPCHK(ee__);                   \
    }

static inline float* blk(vdnn_net& n, int id) { return id < 0 ? nullptr : (float*)(n.pool + n.plan.blocks[id].offset); }

static vdnn_status_t run_fwd(vdnn_net& n, const Op& o) {
    const Layer& l = n.layers[o.layer];
    int C, H, W;
    shape_of(n, l.inputs[0], &C, &H, &W);
    const int N = n.batch;
    float* x = blk(n, o.in_blocks[0]);
    float* y = blk(n, o.out_block);
    const size_t wsb0 = o.ws_block >= 0 ? n.plan.blocks[o.ws_block].bytes : 0;  // no block: the memory-optimal algorithm runs
    switch (l.type) {
        case VDNN_CONV:
            HIPCHK(conv_fwd(x, blk(n, n.plan.w_block[o.layer]), y, blk(n, o.ws_block), wsb0, N, C, H, W, l.out, l.k, l.k, l.stride, l.pad,
                            fold_fwd(n, o.layer) ? 1 : 0, o.kern[0], n.sc));
            break;
        case VDNN_RELU:
            if (l.fwd_folded_into >= 0 && fold_fwd(n, l.fwd_folded_into)) break;  // done in the conv's epilogue
            HIPCHK(relu_fwd(y, n.B(l.buf).count, n.sc));
            break;
        case VDNN_MAXPOOL: HIPCHK(maxpool_fwd(x, y, N, C, H, W, l.k, l.stride, l.pad, n.sc)); break;
        case VDNN_AVGPOOL: HIPCHK(avgpool_fwd(x, y, N, C, H, W, l.k, l.stride, l.pad, n.sc)); break;
        case VDNN_FC: {
            const size_t wsb = o.ws_block >= 0 ? n.plan.blocks[o.ws_block].bytes : 0;
            HIPCHK(fc_fwd(x, blk(n, n.plan.w_block[o.layer]), y, blk(n, o.ws_block), wsb, N, C * H * W, l.out, n.sc));
            break;
        }
        case VDNN_CONCAT: {
            int coff = 0;
            for (size_t k = 0; k < l.inputs.size(); ++k) {
                int c2, h2, w2;
                shape_of(n, l.inputs[k], &c2, &h2, &w2);
                HIPCHK(concat_copy(blk(n, o.in_blocks[k]), y, N, c2, l.C, coff, H * W, 1, n.sc));
                coff += c2;
            }
            break;
        }
        case VDNN_SOFTMAX_CE:
            // the loss block is 256 bytes: the loss in its first word, the count of out-of-range labels in its second
            HIPCHK(softmax_ce_fwd(x, (const int32_t*)blk(n, n.plan.labels_block), blk(n, n.plan.loss_block), (int32_t*)blk(n, n.plan.loss_block) + 1, N,
                                  C * H * W, n.sc));
            break;
    }
    return VDNN_OK;
}

static vdnn_status_t run_bwd(vdnn_net& n, const Op& o) {
    const Layer& l = n.layers[o.layer];
    int C, H, W;
    shape_of(n, l.inputs[0], &C, &H, &W);
    const int N = n.batch;
    float* x = blk(n, o.in_blocks[0]);
    float* dy = blk(n, o.gin_block);
    float* dx = o.gout_blocks.empty() ? nullptr : blk(n, o.gout_blocks[0]);
    const size_t wsb = o.ws_block >= 0 ? n.plan.blocks[o.ws_block].bytes : 0;
    switch (l.type) {
        case VDNN_CONV:
            HIPCHK(conv_bwd_filter(x, dy, blk(n, n.plan.dw_block[o.layer]), blk(n, o.ws_block), wsb, N, C, H, W, l.out, l.k, l.k, l.stride, l.pad, o.kern[2], n.sc));
            if (dx) HIPCHK(conv_bwd_data(dy, blk(n, n.plan.w_block[o.layer]), dx, blk(n, o.ws_block), wsb, N, C, H, W, l.out, l.k, l.k, l.stride, l.pad,
                                         fold_bwd(n, o.layer) ? x : nullptr, o.kern[1], n.sc));
            break;
        case VDNN_RELU:
            if (l.bwd_folded_into >= 0 && fold_bwd(n, l.bwd_folded_into)) break;  // done in the reader's dX store
            HIPCHK(relu_bwd(blk(n, o.out_block), dy, n.B(l.buf).count, n.sc));
            break;
        case VDNN_MAXPOOL: if (dx) HIPCHK(maxpool_bwd(x, dy, dx, N, C, H, W, l.k, l.stride, l.pad, fold_bwd(n, o.layer) ? 1 : 0, n.sc)); break;
        case VDNN_AVGPOOL: if (dx) HIPCHK(avgpool_bwd(dy, dx, N, C, H, W, l.k, l.stride, l.pad, n.sc)); break;
        case VDNN_FC:
            HIPCHK(fc_bwd_filter(x, dy, blk(n, n.plan.dw_block[o.layer]), blk(n, o.ws_block), wsb, N, C * H * W, l.out, n.sc));
            if (dx) HIPCHK(fc_bwd_data(dy, blk(n, n.plan.w_block[o.layer]), dx, blk(n, o.ws_block), wsb, N, C * H * W, l.out, n.sc));
            break;
        case VDNN_CONCAT: {
            int coff = 0;
            for (size_t k = 0; k < l.inputs.size(); ++k) {
                int c2, h2, w2;
                shape_of(n, l.inputs[k], &c2, &h2, &w2);
                if (o.gout_blocks[k] >= 0) HIPCHK(concat_copy(dy, blk(n, o.gout_blocks[k]), N, c2, l.C, coff, H * W, 0, n.sc));
                coff += c2;
            }
            break;
        }
        case VDNN_SOFTMAX_CE:
            if (dx) HIPCHK(softmax_ce_bwd(x, (const int32_t*)blk(n, n.plan.labels_block), dx, N, C * H * W, n.sc));
            break;
    }
    for (size_t k = 0; k < o.gacc_blocks.size(); ++k)
        if (o.gacc_blocks[k] >= 0) HIPCHK(add_inplace(blk(n, o.gacc_blocks[k]), blk(n, o.gout_blocks[k]), n.B(buf_of(n, l.inputs[k])).count, n.sc));
    return VDNN_OK;
}

// Replays ops [first, last) of the plan.
static vdnn_status_t run_ops(vdnn_net& n, int first, int last, const float* input, const int32_t* labels) {
    Plan& p = n.plan;
    constexpr int kSlots = 33;  // per block: the whole block, or up to 32 pieces
    if (n.copy_done_event.size() != p.blocks.size() * kSlots) n.copy_done_event.assign(p.blocks.size() * kSlots, -1);
    for (int t = first; t < last; ++t) {
        const Op& o = p.ops[t];
        switch (o.kind) {
            case OP_SAMPLE:
                if (n.time_layers) {
                    NEWEV(e);
                    HIPCHK(hipEventRecord(n.events[e], n.sc));
                    n.layer_marks.push_back({o.layer, e});
                }
                break;
            case OP_ALLOC:
            case OP_FREE:
                break;  // placement is static: nothing to do at run time
            case OP_LOAD_INPUT:
                HIPCHK(hipMemcpyAsync(blk(n, o.out_block), input, n.B(-1).count * 4, hipMemcpyDeviceToDevice, n.sc));
                HIPCHK(hipMemcpyAsync(blk(n, p.labels_block), labels, (size_t)n.batch * 4, hipMemcpyDeviceToDevice, n.sc));
                break;
            case OP_OFFLOAD:
            case OP_PREFETCH:
            case OP_ONDEMAND: {
                // The copy may start once everything enqueued so far on the compute stream has finished:
                // for an offload that is the producer of X; for a fetch it covers the last users of whatever
                // occupied the destination's address range before.  Pieces of one block that are issued in a
                // row share that edge (nothing was enqueued on the compute stream in between) and are timed
                // as one transfer, which keeps the number of events per step low.
                int prev = t - 1;
                while (prev >= first && (p.ops[prev].kind == OP_ALLOC || p.ops[prev].kind == OP_FREE || p.ops[prev].kind == OP_SAMPLE)) --prev;  // these enqueue nothing
                const bool follows = prev >= first && p.ops[prev].kind == o.kind && p.ops[prev].block == o.block && o.kind != OP_ONDEMAND;
                // Offloads run on the memory stream, fetches on a stream of their own: the link carries both directions at
                // once, and an offload that is still on its way when backward propagation starts does not hold up the first
                // fetches.  (A fetch of X never overtakes the offload of X: its block is allocated after the release of the
                // forward copy, which the compute stream waited for, and the edge below orders the fetch behind that.)
                const hipStream_t cs = o.kind == OP_OFFLOAD || !n.sf ? n.sm : n.sf;
                int e_ready = -1, e0 = -1;
                if (!follows) {
                    NEWEV(er);
                    e_ready = er;
                    HIPCHK(hipEventRecord(n.events[e_ready], n.sc));
                    HIPCHK(hipStreamWaitEvent(cs, n.events[e_ready], 0));
                    NEWEV(es);
                    e0 = es;
                    HIPCHK(hipEventRecord(n.events[e0], cs));
                }
                NEWEV(e1);
                const Block& b = p.blocks[o.block];
                const size_t bytes = o.part < 0 ? b.raw : b.piece_raw(o.part);
                const size_t shift = o.part < 0 ? 0 : (size_t)o.part * b.part_bytes;
                char* host = n.pinned + b.host_off + shift;
                char* dev = (char*)blk(n, o.block) + shift;
                if (bytes) {
                    if (o.kind == OP_OFFLOAD) HIPCHK(hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, cs));
                    else HIPCHK(hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, cs));
                }
                HIPCHK(hipEventRecord(n.events[e1], cs));
                if (follows) { n.copies.back().e1 = e1; n.copies.back().bytes += bytes; }
                else n.copies.push_back({e0, e1, bytes, o.kind == OP_OFFLOAD ? 0 : 1});
                n.copy_done_event[(size_t)o.block * kSlots + o.part + 1] = e1;
                if (o.kind == OP_ONDEMAND) {
                    n.stalls.push_back({e_ready, e1});
                    HIPCHK(hipStreamWaitEvent(n.sc, n.events[e1], 0));
                }
                break;
            }
            case OP_WAIT_COPY: {
                const int e1 = n.copy_done_event[(size_t)o.block * kSlots + o.part + 1];
                if (e1 < 0) { n.err = "internal: wait for a copy that was never issued"; return VDNN_ERR_STATE; }
                // consecutive waits (pieces of one block) are timed as one stall: from here to the last copy awaited
                int prev = t - 1;
                while (prev >= first && (p.ops[prev].kind == OP_ALLOC || p.ops[prev].kind == OP_FREE || p.ops[prev].kind == OP_SAMPLE)) --prev;  // these enqueue nothing
                if (prev >= first && p.ops[prev].kind == OP_WAIT_COPY && !n.stalls.empty()) n.stalls.back().e_copy = e1;
                else {
                    NEWEV(e_here);
                    HIPCHK(hipEventRecord(n.events[e_here], n.sc));
                    n.stalls.push_back({e_here, e1});
                }
                HIPCHK(hipStreamWaitEvent(n.sc, n.events[e1], 0));
                break;
            }
            case OP_FWD: {
                vdnn_status_t s = run_fwd(n, o);
                if (s != VDNN_OK) return s;
                if (n.cap_out[o.layer]) {
                    const Layer& l = n.layers[o.layer];
                    HIPCHK(hipStreamSynchronize(n.sc));
                    if (l.type == VDNN_SOFTMAX_CE) HIPCHK(hipMemcpy(n.cap_out[o.layer], blk(n, p.loss_block), 4, hipMemcpyDeviceToHost));
                    else HIPCHK(hipMemcpy(n.cap_out[o.layer], blk(n, o.out_block), n.B(l.buf).count * 4, hipMemcpyDeviceToHost));
                }
                break;
            }
            case OP_BWD: {
                if (n.cap_grad[o.layer] && o.gin_block >= 0) {
                    HIPCHK(hipStreamSynchronize(n.sc));
                    HIPCHK(hipMemcpy(n.cap_grad[o.layer], blk(n, o.gin_block), n.B(n.layers[o.layer].buf).count * 4, hipMemcpyDeviceToHost));
                }
                vdnn_status_t s = run_bwd(n, o);
                if (s != VDNN_OK) return s;
                break;
            }
        }
    }
    return VDNN_OK;
}

// Pass time and per-layer times after each pass; transfer and stall times after backward propagation, when every copy of
// the step (offloads may still be in flight when forward propagation ends) has completed.
static vdnn_status_t finish_timing(vdnn_net& n, bool bwd) {
    float ms = 0.f;
    if (!bwd) {
        HIPCHK(hipEventElapsedTime(&ms, n.events[n.ev_f0], n.events[n.ev_f1]));
        n.fwd_ms = ms;
    } else {
        HIPCHK(hipEventElapsedTime(&ms, n.events[n.ev_b0], n.events[n.ev_b1]));
        n.bwd_ms = ms;
    }
    if (n.time_layers) {  // a layer's time runs from its start to the start of the next one (or the end of the pass)
        std::vector<float>& out = bwd ? n.layer_bwd_ms : n.layer_fwd_ms;
        out.assign(n.layers.size(), 0.f);
        for (size_t i = 0; i < n.layer_marks.size(); ++i) {
            const int e_next = i + 1 < n.layer_marks.size() ? n.layer_marks[i + 1].second : (bwd ? n.ev_b1 : n.ev_f1);
            HIPCHK(hipEventElapsedTime(&ms, n.events[n.layer_marks[i].second], n.events[e_next]));
            out[n.layer_marks[i].first] = ms;
        }
    }
    n.layer_marks.clear();
    if (!bwd) return VDNN_OK;
    n.stall_ms = n.d2h_ms = n.h2d_ms = 0;
    for (auto& c : n.copies) {
        HIPCHK(hipEventElapsedTime(&ms, n.events[c.e0], n.events[c.e1]));
        (c.dir == 0 ? n.d2h_ms : n.h2d_ms) += ms;
    }
    for (auto& s : n.stalls) {
        hipError_t e = hipEventElapsedTime(&ms, n.events[s.e_compute], n.events[s.e_copy]);
        if (e == hipSuccess && ms > 0.f) n.stall_ms += ms;
        else (void)hipGetLastError();
    }
    n.copies.clear();
    n.stalls.clear();
    return VDNN_OK;
}

// ---------------------------------------------------------------------------------------------
// profiling passes (Section 3.3, "Dynamic vDNN": the layer-wise times of every algorithm are measured on the GPU
// before the policy is chosen)
// ---------------------------------------------------------------------------------------------
// Mean time of `reps` launches of `launch` on the compute stream after one warm-up launch.
template <class F>
static vdnn_status_t time_launches(vdnn_net& n, int reps, float* ms_out, F launch, float give_up_ms = 0.f) {
    NEWEV(e0);
    NEWEV(e1);
    // the warm-up launch is timed too: a kernel that takes more than give_up_ms (> 0) in it is hopeless against what has
    // been measured already, and is not repeated (the gather kernel's unsplit backward-filter runs for most of a second
    // on a large layer)
    HIPCHK(hipEventRecord(n.events[e0], n.sc));
    hipError_t e = launch();
    if (e != hipSuccess) { n.err = fmt("profile: launch failed: %s", hipGetErrorString(e)); (void)hipGetLastError(); n.events_used -= 2; return VDNN_ERR_HIP; }
    HIPCHK(hipEventRecord(n.events[e1], n.sc));
    HIPCHK(hipStreamSynchronize(n.sc));
    float first_ms = 0.f;
    HIPCHK(hipEventElapsedTime(&first_ms, n.events[e0], n.events[e1]));
    if (give_up_ms > 0.f && first_ms > give_up_ms) {
        *ms_out = first_ms;
        n.events_used -= 2;
        return VDNN_OK;
    }
    HIPCHK(hipEventRecord(n.events[e0], n.sc));
    for (int r = 0; r < reps; ++r) {
        e = launch();
        if (e != hipSuccess) { n.err = fmt("profile: launch failed: %s", hipGetErrorString(e)); (void)hipGetLastError(); return VDNN_ERR_HIP; }
    }
    HIPCHK(hipEventRecord(n.events[e1], n.sc));
    HIPCHK(hipStreamSynchronize(n.sc));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, n.events[e0], n.events[e1]));
    *ms_out = ms / (float)reps;
    n.events_used -= 2;
    return VDNN_OK;
}

// Every layer runs alone on zero-filled tensors laid out in the transient part of the pool: forward and backward computation
// as a planned step would launch them, and for CONV layers every kernel that applies, pass by pass.  A layer whose tensors
// do not fit the pool by themselves stays unmeasured (it could not run under this budget either).
static vdnn_status_t profile_layers(vdnn_net& n, int reps) {
    const int L = (int)n.layers.size();
    const Plan saved = n.plan;
    const size_t base = saved.persistent, room = n.pool_bytes - base;
    HIPCHK(hipMemsetAsync(n.pool + base, 0, room, n.sc));
    HIPCHK(hipMemsetAsync(blk(n, saved.labels_block), 0, (size_t)n.batch * 4, n.sc));
    n.profile.assign(L, LayerProfile());
    vdnn_status_t status = VDNN_OK;
    for (int i = 0; i < L && status == VDNN_OK; ++i) {
        const Layer& l = n.layers[i];
        LayerProfile& pr = n.profile[i];
        // a scratch plan: the persistent blocks of the real one, then this layer's tensors one after the other
        Plan q;
        q.ok = true;
        for (const Block& pb : saved.blocks) {  // the persistent blocks come first in every plan
            if (!pb.persistent) break;
            q.blocks.push_back(pb);
        }
        q.w_block = saved.w_block; q.dw_block = saved.dw_block; q.labels_block = saved.labels_block; q.loss_block = saved.loss_block;
        q.persistent = saved.persistent;
        size_t off = base;
        auto add = [&](size_t bytes) {
            Block b;
            b.raw = bytes; b.bytes = align_up(std::max<size_t>(bytes, 1)); b.offset = off;
            off += b.bytes;
            q.blocks.push_back(b);
            return (int)q.blocks.size() - 1;
        };
        Op f, b;
        f.kind = OP_FWD; b.kind = OP_BWD;
        f.layer = b.layer = i;
        const size_t out_bytes = l.type == VDNN_SOFTMAX_CE ? 0 : n.B(l.buf).count * 4;
        for (int src : l.inputs) {
            const int bb = buf_of(n, src);
            const int x = add(n.B(bb).count * 4);
            f.in_blocks.push_back(x);
            b.in_blocks.push_back(x);
            b.gout_blocks.push_back(bb >= 0 && !in_place(l.type) ? add(n.B(bb).count * 4) : -1);
            b.gacc_blocks.push_back(-1);
        }
        if (in_place(l.type)) { f.out_block = b.out_block = f.in_blocks[0]; b.gin_block = add(out_bytes); }
        else if (l.type != VDNN_SOFTMAX_CE) { f.out_block = b.out_block = add(out_bytes); b.gin_block = add(out_bytes); }
        const size_t ws_off = off;
        if (off - base > room) continue;  // does not fit by itself
        n.plan = q;
        if (l.type == VDNN_CONV) {
            int C, H, W;
            shape_of(n, l.inputs[0], &C, &H, &W);
            const int N = n.batch;
            float* x = blk(n, f.in_blocks[0]);
            float* y = blk(n, f.out_block);
            float* dy = blk(n, b.gin_block);
            float* dx = b.gout_blocks[0] >= 0 ? blk(n, b.gout_blocks[0]) : nullptr;
            float* w = blk(n, q.w_block[i]);
            float* dw = blk(n, q.dw_block[i]);
            void* ws = n.pool + ws_off;
            for (int pass = 0; pass < 3 && status == VDNN_OK; ++pass) {
                if (pass == kPassBwdData && !dx) continue;
                float best = -1.f;
                for (int k = kNumKernels - 1; k >= 0 && status == VDNN_OK; --k) {   // the kernels expected fastest first
                    const size_t need = conv_workspace(pass, k, N, C, H, W, l.out, l.k, l.k, l.stride, l.pad);
                    if (need == kNoKernel || ws_off - base + align_up(need) > room) continue;
                    status = time_launches(n, reps, &pr.conv[pass][k], [&]() {
                        if (pass == kPassFwd) return conv_fwd(x, w, y, ws, need, N, C, H, W, l.out, l.k, l.k, l.stride, l.pad, fold_fwd(n, i) ? 1 : 0, k, n.sc);
                        if (pass == kPassBwdData) return conv_bwd_data(dy, w, dx, ws, need, N, C, H, W, l.out, l.k, l.k, l.stride, l.pad, fold_bwd(n, i) ? x : nullptr, k, n.sc);
                        return conv_bwd_filter(x, dy, dw, ws, need, N, C, H, W, l.out, l.k, l.k, l.stride, l.pad, k, n.sc);
                    }, best > 0.f ? std::max(8.f * best, 20.f) : 0.f);
                    if (status == VDNN_OK && (best < 0.f || pr.conv[pass][k] < best)) best = pr.conv[pass][k];
                }
            }
        } else {
            const std::vector<KernelOption>& of = n.options_fwd[i];
            const std::vector<KernelOption>& ob = n.options_bwd[i];
            const size_t wsf = of.empty() ? 0 : of[0].ws, wsb = ob.empty() ? 0 : ob[0].ws;
            if (ws_off - base + align_up(std::max(wsf, wsb)) > room) { n.plan = saved; continue; }
            if (wsf) { f.ws_block = add(wsf); off = ws_off; }
            if (wsb) { b.ws_block = add(wsb); off = ws_off; }
            n.plan.blocks = q.blocks;
            // a ReLU whose work a neighbouring layer does costs nothing by itself
            const bool fwd_elsewhere = l.type == VDNN_RELU && l.fwd_folded_into >= 0 && fold_fwd(n, l.fwd_folded_into);
            const bool bwd_elsewhere = l.type == VDNN_RELU && l.bwd_folded_into >= 0 && fold_bwd(n, l.bwd_folded_into);
            if (fwd_elsewhere) pr.fwd = 0.f;
            else status = time_launches(n, reps, &pr.fwd, [&]() { return run_fwd(n, f) == VDNN_OK ? hipSuccess : hipErrorUnknown; });
            if (status != VDNN_OK) break;
            if (bwd_elsewhere) pr.bwd = 0.f;
            else status = time_launches(n, reps, &pr.bwd, [&]() { return run_bwd(n, b) == VDNN_OK ? hipSuccess : hipErrorUnknown; });
        }
        n.plan = saved;
    }
    n.plan = saved;
    return status;
}

// Rate of the host link in each direction: a 256 MiB block between the pool and pinned host memory on the memory stream.
static vdnn_status_t profile_link(vdnn_net& n) {
    const size_t bytes = std::min<size_t>((size_t)256 << 20, (n.pool_bytes - n.plan.persistent) / kAlign * kAlign);
    if (bytes < ((size_t)1 << 20)) return VDNN_OK;  // a pool this small tells nothing about the link
    char* host = nullptr;
    if (hipHostMalloc((void**)&host, bytes, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); n.err = "profile: no pinned host memory for the link test"; return VDNN_ERR_OOM_HOST; }
    char* dev = n.pool + n.plan.persistent;
    vdnn_status_t status = VDNN_OK;
    for (int dir = 0; dir < 2 && status == VDNN_OK; ++dir) {
        hipError_t e = hipSuccess;
        float ms = 0.f;
        int e0 = -1, e1 = -1;
        { hipError_t ee = hipSuccess; e0 = new_event(n, &ee); e1 = e0 >= 0 ? new_event(n, &ee) : -1; if (e1 < 0) { e = ee; } }
        for (int r = 0; r < 3 && e == hipSuccess; ++r) {  // the first copy warms the path up; the last two are timed
            if (r == 1) e = hipEventRecord(n.events[e0], n.sm);
            if (e == hipSuccess) e = dir == 0 ? hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, n.sm) : hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, n.sm);
        }
        if (e == hipSuccess) e = hipEventRecord(n.events[e1], n.sm);
        if (e == hipSuccess) e = hipStreamSynchronize(n.sm);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, n.events[e0], n.events[e1]);
        n.events_used -= (e0 >= 0) + (e1 >= 0);
        if (e != hipSuccess) { n.err = fmt("profile: link test failed: %s", hipGetErrorString(e)); (void)hipGetLastError(); status = VDNN_ERR_HIP; break; }
        (dir == 0 ? n.link_d2h_gbps : n.link_h2d_gbps) = ms > 0.f ? 2.0 * (double)bytes / (ms * 1e6) : 0.0;
    }
    (void)hipHostFree(host);
    return status;
}

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" {

vdnn_status_t vdnn_create(const vdnn_net_desc_t* desc, size_t gpu_mem_budget, vdnn_net_t** out) {
    if (!desc || !out) return VDNN_ERR_INVALID_ARG;
    vdnn_net* n = new (std::nothrow) vdnn_net();
    if (!n) return VDNN_ERR_OOM_HOST;
    std::string err;
    vdnn_status_t s = build_graph(*n, desc, err);
    if (s != VDNN_OK) { delete n; return s; }
    n->budget = gpu_mem_budget;
    build_kernel_options(*n);
    n->baseline = baseline_bytes(*n);
    s = plan_policy(*n, VDNN_POLICY_NONE);
    // A network that does not fit without offloading is still a valid object: the caller is
    // expected to pick a policy next.  The plan stays invalid until one fits.
    (void)s;
    *out = n;
    return VDNN_OK;
}

vdnn_status_t vdnn_set_conv_algo(vdnn_net_t* n, vdnn_conv_algo_t algo) {
    if (!n || algo < VDNN_ALGO_PERF || algo > VDNN_ALGO_GREEDY) return VDNN_ERR_INVALID_ARG;
    n->static_algo = algo;
    return VDNN_OK;
}

vdnn_status_t vdnn_set_winograd(vdnn_net_t* n, int32_t enabled) {
    if (!n) return VDNN_ERR_INVALID_ARG;
    if (enabled < 0 || enabled > 2) return VDNN_ERR_INVALID_ARG;
    n->winograd = enabled;
    build_kernel_options(*n);
    return VDNN_OK;
}

vdnn_status_t vdnn_set_policy(vdnn_net_t* n, vdnn_policy_t policy) {
    if (!n || policy < VDNN_POLICY_NONE || policy > VDNN_POLICY_FIT) return VDNN_ERR_INVALID_ARG;
    n->fwd_done = false;
    return plan_policy(*n, policy);
}

vdnn_status_t vdnn_set_offload_set(vdnn_net_t* np, const int32_t* buffers, size_t count, int32_t window_fill_pm, int32_t window_fill_bwd_pm) {
    if (!np || (count && !buffers) || window_fill_pm < 0 || window_fill_pm > 1000 || window_fill_bwd_pm < 0 || window_fill_bwd_pm > 1000)
        return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    const int L = (int)n.layers.size();
    std::vector<char> set(L + 1, 0);
    for (size_t i = 0; i < count; ++i) {
        const int b = buffers[i];
        // what ALL would offload, and (Section 3, opening: the same idea applies to the classification layers) the X of FC layers
        bool ok = b >= -1 && b < L && n.B(b).count && !n.B(b).bwd_users.empty();
        if (ok && !selected(n, b, VDNN_POLICY_ALL)) {
            ok = false;
            for (int r : n.B(b).readers) ok |= n.layers[r].type == VDNN_FC;
        }
        if (!ok) {
            n.err = fmt("set_offload_set: %d is not a feature map that a CONV, POOL or FC layer reads and backward propagation needs", b);
            return VDNN_ERR_INVALID_ARG;
        }
        set[b + 1] = 1;
    }
    n.fwd_done = false;
    Plan p;
    compile_plan(n, VDNN_POLICY_CUSTOM, n.static_algo, p, &set, true, window_fill_pm, window_fill_bwd_pm);
    if (!p.ok) { n.err = p.fail_why; return VDNN_ERR_OOM_DEVICE; }
    n.plan = p; n.policy = n.effective = VDNN_POLICY_CUSTOM;
    return VDNN_OK;
}

vdnn_status_t vdnn_set_window_part(vdnn_net_t* n, size_t part_bytes) {
    if (!n) return VDNN_ERR_INVALID_ARG;
    n->part_bytes = part_bytes;
    return VDNN_OK;
}

vdnn_status_t vdnn_get_offload_set(const vdnn_net_t* n, int32_t* buffers, size_t cap, size_t* count) {
    if (!n || !count) return VDNN_ERR_INVALID_ARG;
    size_t k = 0;
    for (size_t i = 0; i < n->plan.offload_set.size(); ++i) {
        if (!n->plan.ok || !n->plan.offload_set[i]) continue;
        if (buffers && k < cap) buffers[k] = (int32_t)i - 1;
        ++k;
    }
    *count = k;
    return VDNN_OK;
}

vdnn_status_t vdnn_attach_device(vdnn_net_t* np, void* pool_base, size_t pool_bytes, void* stream_compute, void* stream_memory) {
    if (!np || !pool_base || !stream_compute || !stream_memory || stream_compute == stream_memory) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    if (((uintptr_t)pool_base) % kAlign) { n.err = "pool base must be 256-byte aligned"; return VDNN_ERR_INVALID_ARG; }
    if (n.weights_set) { n.err = "attach the device pool before setting weights"; return VDNN_ERR_STATE; }
    if (n.own_pool && n.pool) { HIPCHK(hipFree(n.pool)); }
    n.pool = (char*)pool_base; n.pool_bytes = pool_bytes; n.own_pool = false;
    if (n.own_streams) { HIPCHK(hipStreamDestroy(n.sc)); HIPCHK(hipStreamDestroy(n.sm)); }
    n.sc = (hipStream_t)stream_compute; n.sm = (hipStream_t)stream_memory;
    n.have_streams = true; n.own_streams = false;
    return VDNN_OK;
}

size_t vdnn_weight_count(const vdnn_net_t* n, int layer) {
    if (!n || layer < 0 || layer >= (int)n->layers.size()) return 0;
    return n->layers[layer].wcount;
}

size_t vdnn_output_count(const vdnn_net_t* n, int layer) {
    if (!n || layer < 0 || layer >= (int)n->layers.size()) return 0;
    const Layer& l = n->layers[layer];
    return l.type == VDNN_SOFTMAX_CE ? 1 : (size_t)n->batch * l.C * l.H * l.W;
}

vdnn_status_t vdnn_set_weights(vdnn_net_t* np, int layer, const float* w, size_t count) {
    if (!np || !w) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    if (layer < 0 || layer >= (int)n.layers.size() || !n.layers[layer].wcount || n.layers[layer].wcount != count) {
        n.err = "set_weights: wrong layer or count";
        return VDNN_ERR_INVALID_ARG;
    }
    vdnn_status_t s = ensure_device(n);
    if (s != VDNN_OK) return s;
    HIPCHK(hipMemcpy(blk(n, n.plan.w_block[layer]), w, count * 4, hipMemcpyHostToDevice));
    n.weights_set = true;
    return VDNN_OK;
}

vdnn_status_t vdnn_get_weight_grad(vdnn_net_t* np, int layer, float* dw, size_t count) {
    if (!np || !dw) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    if (layer < 0 || layer >= (int)n.layers.size() || !n.layers[layer].wcount || n.layers[layer].wcount != count) {
        n.err = "get_weight_grad: wrong layer or count";
        return VDNN_ERR_INVALID_ARG;
    }
    if (!n.pool) { n.err = "no step has run"; return VDNN_ERR_STATE; }
    HIPCHK(hipStreamSynchronize(n.sc));
    HIPCHK(hipMemcpy(dw, blk(n, n.plan.dw_block[layer]), count * 4, hipMemcpyDeviceToHost));
    return VDNN_OK;
}

vdnn_status_t vdnn_get_weights(vdnn_net_t* np, int layer, float* w, size_t count) {
    if (!np || !w) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    if (layer < 0 || layer >= (int)n.layers.size() || !n.layers[layer].wcount || n.layers[layer].wcount != count) {
        n.err = "get_weights: wrong layer or count";
        return VDNN_ERR_INVALID_ARG;
    }
    if (!n.pool) { n.err = "weights were never set"; return VDNN_ERR_STATE; }
    HIPCHK(hipStreamSynchronize(n.sc));
    HIPCHK(hipMemcpy(w, blk(n, n.plan.w_block[layer]), count * 4, hipMemcpyDeviceToHost));
    return VDNN_OK;
}

vdnn_status_t vdnn_sgd_step(vdnn_net_t* np, float learning_rate) {
    if (!np) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    if (!n.pool || !n.have_streams || !n.plan.ok) { n.err = "sgd_step before any backward pass"; return VDNN_ERR_STATE; }
    for (size_t i = 0; i < n.layers.size(); ++i)
        if (n.layers[i].wcount) HIPCHK(sgd_update(blk(n, n.plan.w_block[i]), blk(n, n.plan.dw_block[i]), learning_rate, n.layers[i].wcount, n.sc));
    HIPCHK(hipStreamSynchronize(n.sc));
    return VDNN_OK;
}

vdnn_status_t vdnn_get_output(vdnn_net_t* np, int layer, float* dst, size_t count) {
    if (!np || !dst) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    const int L = (int)n.layers.size();
    if (layer == -1) layer = n.layers[L - 1].inputs[0];  // the logits: what the loss layer reads
    if (layer < 0 || layer >= L || n.layers[layer].type == VDNN_SOFTMAX_CE || count != vdnn_output_count(np, layer)) {
        n.err = "get_output: wrong layer or count";
        return VDNN_ERR_INVALID_ARG;
    }
    if (!n.fwd_done) { n.err = "get_output: only between a completed forward pass and the backward pass that follows it"; return VDNN_ERR_STATE; }
    const int b = n.layers[layer].buf;
    const Plan& p = n.plan;
    // where the feature map is at the end of forward propagation: in the pinned arena when the plan offloads it, else in the
    // block that is still live when backward propagation starts
    int dev_block = -1, host_block = -1;
    for (int t = p.first_fwd_op; t < p.first_bwd_op; ++t)
        if (p.ops[t].kind == OP_OFFLOAD && p.ops[t].buf == b) host_block = p.ops[t].block;
    for (int id = 0; id < (int)p.blocks.size() && host_block < 0; ++id)
        if (p.blocks[id].buf == b && !p.blocks[id].persistent && p.blocks[id].t0 < p.first_bwd_op && p.blocks[id].t1 > p.first_bwd_op) dev_block = id;
    if (host_block >= 0) {
        HIPCHK(hipStreamSynchronize(n.sm));   // the offload may still be on its way
        memcpy(dst, n.pinned + p.blocks[host_block].host_off, count * 4);
    }
    else if (dev_block >= 0) HIPCHK(hipMemcpy(dst, blk(n, dev_block), count * 4, hipMemcpyDeviceToHost));
    else { n.err = fmt("get_output: the output of layer %d was released during forward propagation (no backward computation reads it)", layer); return VDNN_ERR_STATE; }
    return VDNN_OK;
}

vdnn_status_t vdnn_capture_output(vdnn_net_t* n, int layer, float* dst) {
    if (!n || layer < 0 || layer >= (int)n->layers.size()) return VDNN_ERR_INVALID_ARG;
    n->cap_out[layer] = dst;
    return VDNN_OK;
}

vdnn_status_t vdnn_capture_grad(vdnn_net_t* n, int layer, float* dst) {
    if (!n || layer < 0 || layer >= (int)n->layers.size()) return VDNN_ERR_INVALID_ARG;
    n->cap_grad[layer] = dst;
    return VDNN_OK;
}

vdnn_status_t vdnn_forward(vdnn_net_t* np, const float* input, const int32_t* labels, float* loss_out) {
    if (!np || !input || !labels) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    vdnn_status_t s = ensure_device(n);
    if (s != VDNN_OK) return s;
    n.fwd_done = false;
    // copies of a step that was abandoned after its forward pass may still be reading the pool this pass is about to overwrite
    HIPCHK(hipStreamSynchronize(n.sm));
    if (n.sf) HIPCHK(hipStreamSynchronize(n.sf));
    n.events_used = 0;
    n.copies.clear();
    n.stalls.clear();
    n.layer_marks.clear();
    { NEWEV(e); n.ev_f0 = e; }
    { NEWEV(e); n.ev_f1 = e; }
    HIPCHK(hipEventRecord(n.events[n.ev_f0], n.sc));
    s = run_ops(n, n.plan.first_fwd_op, n.plan.first_bwd_op, input, labels);
    if (s != VDNN_OK) { (void)hipDeviceSynchronize(); return s; }
    HIPCHK(hipEventRecord(n.events[n.ev_f1], n.sc));
    // the forward COMPUTATION has completed when this returns; offloads whose release the plan has postponed into backward
    // propagation (transfer windows) may still be on their way to the host
    HIPCHK(hipStreamSynchronize(n.sc));
    struct { float loss; int32_t bad_labels; } res = {0.f, 0};
    HIPCHK(hipMemcpy(&res, blk(n, n.plan.loss_block), sizeof res, hipMemcpyDeviceToHost));
    const float loss = res.loss;
    s = finish_timing(n, false);
    if (s != VDNN_OK) return s;
    if (res.bad_labels) {
        n.err = fmt("%d of the %d labels are outside [0, classes)", res.bad_labels, n.batch);
        return VDNN_ERR_INVALID_ARG;
    }
    if (loss_out) *loss_out = loss;
    n.fwd_done = true;
    return VDNN_OK;
}

vdnn_status_t vdnn_backward(vdnn_net_t* np) {
    if (!np) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    if (!n.fwd_done) { n.err = "backward without a completed forward"; return VDNN_ERR_STATE; }
    n.fwd_done = false;
    { NEWEV(e); n.ev_b0 = e; }
    { NEWEV(e); n.ev_b1 = e; }
    HIPCHK(hipEventRecord(n.events[n.ev_b0], n.sc));
    vdnn_status_t s = run_ops(n, n.plan.first_bwd_op, (int)n.plan.ops.size(), nullptr, nullptr);
    if (s != VDNN_OK) { (void)hipDeviceSynchronize(); return s; }
    HIPCHK(hipEventRecord(n.events[n.ev_b1], n.sc));
    HIPCHK(hipStreamSynchronize(n.sc));
    HIPCHK(hipStreamSynchronize(n.sm));
    if (n.sf) HIPCHK(hipStreamSynchronize(n.sf));
    return finish_timing(n, true);
}

vdnn_status_t vdnn_mem_stats(const vdnn_net_t* n, vdnn_mem_stats_t* out) {
    if (!n || !out) return VDNN_ERR_INVALID_ARG;
    vdnn_mem_stats_t s;
    memset(&s, 0, sizeof s);
    const Plan& p = n->plan;
    s.budget_bytes = n->budget;
    s.baseline_bytes = n->baseline;
    s.effective_policy = n->effective;
    if (p.ok) {
        s.cur_bytes = p.persistent;
        s.peak_bytes = p.peak;
        s.pool_extent_bytes = p.extent;
        s.persistent_bytes = p.persistent;
        s.avg_bytes_layerstep = p.avg;
        s.offloaded_bytes = p.offloaded;
        s.prefetched_bytes = p.prefetched;
        s.pinned_host_bytes = p.pinned;
        s.workspace_bytes = p.max_ws;
        s.n_offload = p.n_offload;
        s.n_prefetch = p.n_prefetch;
        s.n_ondemand_fetch = p.n_ondemand;
        s.conv_algo = p.algo;
        s.n_memopt_convs = p.n_memopt;
        s.n_winograd_convs = p.n_winograd;
        s.n_downgraded_convs = p.n_downgraded;
        s.window_fill_pm = p.fill_pm;
        s.window_fill_bwd_pm = p.fill_bwd_pm;
    }
    s.fwd_ms = n->fwd_ms; s.bwd_ms = n->bwd_ms; s.stall_ms = n->stall_ms;
    s.d2h_ms = n->d2h_ms; s.h2d_ms = n->h2d_ms;
    s.d2h_gbps = n->d2h_ms > 0 ? (double)p.offloaded / (n->d2h_ms * 1e6) : 0.0;
    s.h2d_gbps = n->h2d_ms > 0 ? (double)p.prefetched / (n->h2d_ms * 1e6) : 0.0;
    *out = s;
    return VDNN_OK;
}

vdnn_status_t vdnn_layer_workspace_options(const vdnn_net_t* n, int layer, int32_t bwd, uint64_t* bytes, size_t cap, size_t* count) {
    if (!n || !count || layer < 0 || layer >= (int)n->layers.size()) return VDNN_ERR_INVALID_ARG;
    const std::vector<KernelOption>& v = (bwd ? n->options_bwd : n->options_fwd)[layer];
    for (size_t k = 0; k < v.size() && k < cap && bytes; ++k) bytes[k] = v[k].ws;
    *count = v.size();
    return VDNN_OK;
}

vdnn_status_t vdnn_layer_kernels(const vdnn_net_t* n, int layer, int32_t kernels[3]) {
    if (!n || !kernels || layer < 0 || layer >= (int)n->layers.size() || n->layers[layer].type != VDNN_CONV) return VDNN_ERR_INVALID_ARG;
    if (!n->plan.ok) return VDNN_ERR_STATE;
    // from the plan's own ops: what the step launches (the layer's lists may have been rebuilt since the plan was made)
    kernels[0] = kernels[1] = kernels[2] = kKernelGather;
    for (const Op& o : n->plan.ops) {
        if (o.layer != layer) continue;
        if (o.kind == OP_FWD) kernels[0] = o.kern[0];
        if (o.kind == OP_BWD) { kernels[1] = o.kern[1]; kernels[2] = o.kern[2]; }
    }
    return VDNN_OK;
}

vdnn_status_t vdnn_set_layer_kernels(vdnn_net_t* np, int layer, const int32_t kernels[3]) {
    if (!np || layer < 0 || layer >= (int)np->layers.size() || np->layers[layer].type != VDNN_CONV) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    if (!kernels) {
        n.pinned_kernels[layer] = -1;
    } else {
        const Layer& l = n.layers[layer];
        int C, H, W;
        shape_of(n, l.inputs[0], &C, &H, &W);
        const bool need_dx = buf_of(n, l.inputs[0]) >= 0;
        for (int pass = 0; pass < 3; ++pass) {
            if (pass == kPassBwdData && !need_dx) continue;
            if (kernels[pass] < 0 || kernels[pass] >= kNumKernels ||
                conv_workspace(pass, kernels[pass], n.batch, C, H, W, l.out, l.k, l.k, l.stride, l.pad) == kNoKernel) {
                n.err = fmt("set_layer_kernels: kernel %d does not apply to pass %d of layer %d", kernels[pass], pass, layer);
                return VDNN_ERR_INVALID_ARG;
            }
        }
        n.pinned_kernels[layer] = kernels[0] | (need_dx ? kernels[1] : 0) << 4 | kernels[2] << 8;
    }
    build_kernel_options(n);
    return VDNN_OK;
}

vdnn_status_t vdnn_profile(vdnn_net_t* np, int32_t repeats) {
    if (!np || repeats < 1 || repeats > 100) return VDNN_ERR_INVALID_ARG;
    vdnn_net& n = *np;
    vdnn_status_t s = ensure_device(n);   // needs a plan that fits: its pool is where the layers run
    if (s != VDNN_OK) return s;
    n.fwd_done = false;
    HIPCHK(hipStreamSynchronize(n.sm));
    if (n.sf) HIPCHK(hipStreamSynchronize(n.sf));
    n.events_used = 0;
    n.copies.clear();
    n.stalls.clear();
    n.layer_marks.clear();
    s = profile_layers(n, repeats);
    if (s == VDNN_OK) s = profile_link(n);
    (void)hipStreamSynchronize(n.sc);
    (void)hipStreamSynchronize(n.sm);
    if (s != VDNN_OK) return s;
    n.profiled = true;
    build_kernel_options(n);
    return VDNN_OK;
}

vdnn_status_t vdnn_set_layer_profile(vdnn_net_t* n, int layer, int32_t pass, int32_t kernel, float ms) {
    if (!n || layer < 0 || layer >= (int)n->layers.size() || pass < 0 || pass > 2 || !(ms >= 0.f)) return VDNN_ERR_INVALID_ARG;
    vdnn::LayerProfile& pr = n->profile[layer];
    if (n->layers[layer].type == VDNN_CONV) {
        if (kernel < 0 || kernel >= kNumKernels) return VDNN_ERR_INVALID_ARG;
        pr.conv[pass][kernel] = ms;
    } else {
        if (pass > 1) return VDNN_ERR_INVALID_ARG;
        (pass == 0 ? pr.fwd : pr.bwd) = ms;
    }
    n->profiled = true;
    build_kernel_options(*n);
    return VDNN_OK;
}

vdnn_status_t vdnn_get_layer_profile(const vdnn_net_t* n, int layer, int32_t pass, int32_t kernel, float* ms) {
    if (!n || !ms || layer < 0 || layer >= (int)n->layers.size() || pass < 0 || pass > 2) return VDNN_ERR_INVALID_ARG;
    const vdnn::LayerProfile& pr = n->profile[layer];
    if (n->layers[layer].type == VDNN_CONV) {
        if (kernel < 0 || kernel >= kNumKernels) return VDNN_ERR_INVALID_ARG;
        *ms = pr.conv[pass][kernel];
    } else {
        if (pass > 1) return VDNN_ERR_INVALID_ARG;
        *ms = pass == 0 ? pr.fwd : pr.bwd;
    }
    return VDNN_OK;
}

vdnn_status_t vdnn_estimate_step_ms(const vdnn_net_t* n, double* ms) {
    if (!n || !ms) return VDNN_ERR_INVALID_ARG;
    if (!n->plan.ok || !n->profiled) return VDNN_ERR_STATE;
    *ms = estimate_step_ms(*n, n->plan);
    return VDNN_OK;
}

vdnn_status_t vdnn_set_link_rate(vdnn_net_t* n, double d2h_gbps, double h2d_gbps) {
    if (!n || !(d2h_gbps > 0.0) || !(h2d_gbps > 0.0)) return VDNN_ERR_INVALID_ARG;
    n->link_d2h_gbps = d2h_gbps; n->link_h2d_gbps = h2d_gbps;
    return VDNN_OK;
}

vdnn_status_t vdnn_get_link_rate(const vdnn_net_t* n, double* d2h_gbps, double* h2d_gbps) {
    if (!n || !d2h_gbps || !h2d_gbps) return VDNN_ERR_INVALID_ARG;
    *d2h_gbps = n->link_d2h_gbps; *h2d_gbps = n->link_h2d_gbps;
    return VDNN_OK;
}

vdnn_status_t vdnn_set_layer_timing(vdnn_net_t* n, int32_t on) {
    if (!n) return VDNN_ERR_INVALID_ARG;
    n->time_layers = on != 0;
    return VDNN_OK;
}

vdnn_status_t vdnn_layer_times(const vdnn_net_t* n, float* fwd_ms, float* bwd_ms, size_t count) {
    if (!n || !fwd_ms || !bwd_ms || count != n->layers.size()) return VDNN_ERR_INVALID_ARG;
    if (n->layer_fwd_ms.size() != count || n->layer_bwd_ms.size() != count) return VDNN_ERR_STATE;
    memcpy(fwd_ms, n->layer_fwd_ms.data(), count * sizeof(float));
    memcpy(bwd_ms, n->layer_bwd_ms.data(), count * sizeof(float));
    return VDNN_OK;
}

vdnn_status_t vdnn_trace(const vdnn_net_t* n, char* buf, size_t cap, size_t* needed) {
    if (!n || !needed) return VDNN_ERR_INVALID_ARG;
    std::string s;
    const Plan& p = n->plan;
    for (const Op& o : p.ops) {
        std::string where = o.phase == 0 ? "create" : fmt("%c%d", o.phase == 1 ? 'F' : 'B', o.layer);
        switch (o.kind) {
            case OP_ALLOC:
            case OP_FREE: {
                const Block& b = p.blocks[o.block];
                const char* what = o.kind == OP_ALLOC ? "alloc" : "free";
                if (o.part < 0) s += fmt("%s %s %s %zu %zu\n", where.c_str(), what, b.tag.c_str(), b.bytes, b.offset);
                else s += fmt("%s %s %s#%d %zu %zu\n", where.c_str(), what, b.tag.c_str(), o.part, b.piece_bytes(o.part), b.offset + (size_t)o.part * b.part_bytes);
                break;
            }
            case OP_OFFLOAD:
            case OP_PREFETCH:
            case OP_ONDEMAND: {
                const Block& b = p.blocks[o.block];
                const char* what = o.kind == OP_OFFLOAD ? "offload" : (o.kind == OP_PREFETCH ? "prefetch" : "ondemand");
                if (o.part < 0) s += fmt("%s %s B%d %zu\n", where.c_str(), what, o.buf, b.raw);
                else s += fmt("%s %s B%d#%d %zu\n", where.c_str(), what, o.buf, o.part, b.piece_raw(o.part));
                break;
            }
            case OP_FWD:
            case OP_BWD: s += fmt("%s compute %s\n", where.c_str(), type_name(n->layers[o.layer].type)); break;
            default: break;
        }
    }
    if (!p.ok && !p.fail_where.empty()) s += "fail " + p.fail_where + "\n";
    *needed = s.size() + 1;
    if (buf && cap) {
        const size_t k = std::min(cap - 1, s.size());
        memcpy(buf, s.data(), k);
        buf[k] = 0;
    }
    return VDNN_OK;
}

const char* vdnn_last_error(const vdnn_net_t* n) { return n ? n->err.c_str() : "null net"; }

void vdnn_destroy(vdnn_net_t* n) {
    if (!n) return;
    if (n->have_streams) { (void)hipStreamSynchronize(n->sc); (void)hipStreamSynchronize(n->sm); }
    if (n->sf) (void)hipStreamSynchronize(n->sf);
    for (hipEvent_t e : n->events) (void)hipEventDestroy(e);
    if (n->own_streams) { (void)hipStreamDestroy(n->sc); (void)hipStreamDestroy(n->sm); }
    if (n->own_pool && n->pool) (void)hipFree(n->pool);
    if (n->pinned) (void)hipHostFree(n->pinned);
    delete n;
}

}  // extern "C"
