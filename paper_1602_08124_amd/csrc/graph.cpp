// Dataflow graph of a network description: validation, shapes, feature-map buffers with their readers,
// ReLU folding links, workspace sizes and the baseline (network-wide) allocation.
#include "manager.h"

#include <algorithm>
#include <cstring>

#include "ops.h"

namespace vdnn {

// ---------------------------------------------------------------------------------------------
// graph
// ---------------------------------------------------------------------------------------------
vdnn_status_t build_graph(vdnn_net& n, const vdnn_net_desc_t* d, std::string& err) {
    if (d->batch <= 0 || d->in_c <= 0 || d->in_h <= 0 || d->in_w <= 0 || d->n_layers <= 0 || !d->layers) {
        err = "bad network dimensions";
        return VDNN_ERR_INVALID_ARG;
    }
    n.batch = d->batch; n.in_c = d->in_c; n.in_h = d->in_h; n.in_w = d->in_w;
    const int L = d->n_layers;
    n.layers.resize(L);
    std::vector<int> n_consumers(L + 1, 0);
    for (int i = 0; i < L; ++i) {
        const vdnn_layer_desc_t& s = d->layers[i];
        Layer& l = n.layers[i];
        l.type = s.type; l.out = s.out_channels; l.k = s.kernel; l.stride = s.stride; l.pad = s.pad;
        if (s.type < 0 || s.type > VDNN_SOFTMAX_CE) { err = fmt("layer %d: unknown type %d", i, s.type); return VDNN_ERR_INVALID_ARG; }
        const int want_min = s.type == VDNN_CONCAT ? 2 : 1, want_max = s.type == VDNN_CONCAT ? VDNN_MAX_INPUTS : 1;
        if (s.n_inputs < want_min || s.n_inputs > want_max) { err = fmt("layer %d: bad number of inputs %d", i, s.n_inputs); return VDNN_ERR_INVALID_ARG; }
        for (int j = 0; j < s.n_inputs; ++j) {
            const int src = s.inputs[j];
            if (src < -1 || src >= i) { err = fmt("layer %d: input %d is not an earlier layer", i, src); return VDNN_ERR_INVALID_ARG; }
            if (src >= 0 && n.layers[src].type == VDNN_SOFTMAX_CE) { err = fmt("layer %d consumes the loss", i); return VDNN_ERR_INVALID_ARG; }
            if (std::find(l.inputs.begin(), l.inputs.end(), src) != l.inputs.end()) { err = fmt("layer %d: duplicate input %d", i, src); return VDNN_ERR_INVALID_ARG; }
            l.inputs.push_back(src);
            n_consumers[src + 1]++;
        }
        int C, H, W;
        shape_of(n, l.inputs[0], &C, &H, &W);
        switch (l.type) {
            case VDNN_CONV:
                if (l.out <= 0 || l.k <= 0 || l.stride <= 0 || l.pad < 0) { err = fmt("layer %d: bad conv geometry", i); return VDNN_ERR_INVALID_ARG; }
                l.C = l.out; l.H = (H + 2 * l.pad - l.k) / l.stride + 1; l.W = (W + 2 * l.pad - l.k) / l.stride + 1;
                if (H + 2 * l.pad < l.k || W + 2 * l.pad < l.k) { err = fmt("layer %d: window larger than image", i); return VDNN_ERR_INVALID_ARG; }
                l.wcount = (size_t)l.out * C * l.k * l.k;
                break;
            case VDNN_MAXPOOL:
            case VDNN_AVGPOOL:
                if (l.k <= 0 || l.stride <= 0 || l.pad < 0 || l.pad >= l.k || H + 2 * l.pad < l.k || W + 2 * l.pad < l.k) { err = fmt("layer %d: bad pool geometry", i); return VDNN_ERR_INVALID_ARG; }
                l.C = C; l.H = (H + 2 * l.pad - l.k) / l.stride + 1; l.W = (W + 2 * l.pad - l.k) / l.stride + 1;
                break;
            case VDNN_FC:
                if (l.out <= 0) { err = fmt("layer %d: bad fc size", i); return VDNN_ERR_INVALID_ARG; }
                l.C = l.out; l.H = 1; l.W = 1;
                l.wcount = (size_t)l.out * C * H * W;
                break;
            case VDNN_CONCAT: {
                int csum = 0;
                for (int src : l.inputs) {
                    int c2, h2, w2;
                    shape_of(n, src, &c2, &h2, &w2);
                    if (h2 != H || w2 != W) { err = fmt("layer %d: concat inputs differ in size", i); return VDNN_ERR_INVALID_ARG; }
                    csum += c2;
                }
                l.C = csum; l.H = H; l.W = W;
                break;
            }
            case VDNN_RELU:
                l.C = C; l.H = H; l.W = W;
                break;
            case VDNN_SOFTMAX_CE:
                if (i != L - 1) { err = "softmax_ce must be the last layer"; return VDNN_ERR_INVALID_ARG; }
                l.C = l.H = l.W = 0;
                break;
        }
        if (l.type != VDNN_SOFTMAX_CE && (l.H <= 0 || l.W <= 0)) { err = fmt("layer %d: empty output", i); return VDNN_ERR_INVALID_ARG; }
        l.buf = in_place(l.type) ? buf_of(n, l.inputs[0]) : i;
    }
    if (n.layers[L - 1].type != VDNN_SOFTMAX_CE) { err = "the last layer must be softmax_ce"; return VDNN_ERR_INVALID_ARG; }
    for (int i = 0; i < L; ++i) {
        if (in_place(n.layers[i].type) && n_consumers[n.layers[i].inputs[0] + 1] != 1) {
            err = fmt("layer %d: an in-place layer must be the only consumer of its input", i);
            return VDNN_ERR_INVALID_ARG;
        }
        if (n.layers[i].type != VDNN_SOFTMAX_CE && n_consumers[i + 1] == 0) { err = fmt("layer %d: output is never consumed", i); return VDNN_ERR_INVALID_ARG; }
    }
    if (n_consumers[0] == 0) { err = "the network input is never consumed"; return VDNN_ERR_INVALID_ARG; }
    n.bufs.assign(L + 1, Buffer());
    for (int b = -1; b < L; ++b) {
        if (b >= 0 && (n.layers[b].buf != b || n.layers[b].type == VDNN_SOFTMAX_CE)) continue;
        Buffer& B = n.B(b);
        shape_of(n, b, &B.C, &B.H, &B.W);
        B.count = (size_t)n.batch * B.C * B.H * B.W;
        if (B.count >= 0x7fffffffULL) { err = fmt("feature map %d has 2^31 or more elements", b); return VDNN_ERR_UNSUPPORTED; }
    }
    for (int i = 0; i < L; ++i) {
        const Layer& l = n.layers[i];
        if (in_place(l.type)) {
            if (l.buf < 0) { err = "an in-place layer cannot overwrite the network input"; return VDNN_ERR_INVALID_ARG; }
            n.B(l.buf).inplace.push_back(i);
        } else {
            for (int src : l.inputs) n.B(buf_of(n, src)).readers.push_back(i);
        }
    }
    for (int b = -1; b < L; ++b) {
        Buffer& B = n.B(b);
        if (!B.count) continue;
        for (int r : B.readers)
            if (needs_x_in_bwd(n.layers[r].type)) B.bwd_users.push_back(r);
        for (int r : B.inplace) B.bwd_users.push_back(r);
        std::sort(B.bwd_users.begin(), B.bwd_users.end());
    }
    // ReLU folding.  Forward: a CONV whose output holds exactly one in-place ReLU applies it in its
    // epilogue.  Backward: when a feature map holds exactly one in-place ReLU and has a single reader
    // that is a CONV or max-POOL layer, that reader masks its dX store with (X > 0), which is the
    // ReLU's backward computation.  Values are identical to running the ReLU kernels separately.
    for (int b = 0; b < L; ++b) {
        Buffer& B = n.B(b);
        if (!B.count || B.inplace.size() != 1) continue;
        const int r = B.inplace[0];
        if (n.layers[b].type == VDNN_CONV) { n.layers[b].relu_after = r; n.layers[r].fwd_folded_into = b; }
        if (B.readers.size() == 1) {
            const int m = B.readers[0];
            if (n.layers[m].type == VDNN_CONV || n.layers[m].type == VDNN_MAXPOOL) { n.layers[m].relu_before = r; n.layers[r].bwd_folded_into = m; }
        }
    }
    n.cap_out.assign(L, nullptr);
    n.cap_grad.assign(L, nullptr);
    return VDNN_OK;
}

// A test hook on the tensors in between switches the folding off for that pair, so that the hook
// still sees the unfused intermediate value.
bool fold_fwd(const vdnn_net& n, int conv) {
    const int r = n.layers[conv].relu_after;
    return r >= 0 && !n.cap_out[conv];
}
bool fold_bwd(const vdnn_net& n, int reader) {
    const int r = n.layers[reader].relu_before;
    return r >= 0 && !n.cap_grad[r];
}

// ---------------------------------------------------------------------------------------------
// how each layer can run: kernels, workspace, cost (Section 2.2: algorithms trade workspace for speed; Section 3.3:
// vDNN_dyn profiles them per layer)
// ---------------------------------------------------------------------------------------------
// Keeps, in ascending cost, the options that a greedy choice could ever take: one that needs at least as much
// workspace as a cheaper one never is.
static void sort_and_prune(std::vector<KernelOption>& v) {
    std::stable_sort(v.begin(), v.end(), [](const KernelOption& a, const KernelOption& b) { return a.cost < b.cost; });
    std::vector<KernelOption> keep;
    for (const KernelOption& o : v)
        if (keep.empty() || o.ws < keep.back().ws) keep.push_back(o);
    v.swap(keep);
}

void build_kernel_options(vdnn_net& n) {
    const int L = (int)n.layers.size();
    n.options_fwd.assign(L, {});
    n.options_bwd.assign(L, {});
    if ((int)n.profile.size() != L) n.profile.assign(L, LayerProfile());
    if ((int)n.pinned_kernels.size() != L) n.pinned_kernels.assign(L, -1);
    for (int i = 0; i < L; ++i) {
        const Layer& l = n.layers[i];
        int C, H, W;
        shape_of(n, l.inputs[0], &C, &H, &W);
        if (l.type == VDNN_FC) {
            const int I = C * H * W;
            const bool need_dx = buf_of(n, l.inputs[0]) >= 0;
            KernelOption f, b;
            f.ws = fc_workspace(n.batch, I, l.out, 0);
            b.ws = std::max(fc_workspace(n.batch, I, l.out, 2), need_dx ? fc_workspace(n.batch, I, l.out, 1) : (size_t)0);
            n.options_fwd[i].push_back(f);
            n.options_bwd[i].push_back(b);
            continue;
        }
        if (l.type != VDNN_CONV) continue;
        const LayerProfile& pr = n.profile[i];
        auto ws_of = [&](int pass, int k) { return conv_workspace(pass, k, n.batch, C, H, W, l.out, l.k, l.k, l.stride, l.pad); };
        // no profile: Winograd, then Winograd on smaller chunks, then the packed-weight kernel, then the gather kernel (measured on the paper's workloads);
        // with one, a kernel that was not measured (its tensors and workspace did not fit the pool together) comes after all that were
        auto cost_of = [&](int pass, int k) {
            if (!n.profiled) return (double)kernel_rank(k);
            return pr.conv[pass][k] >= 0 ? (double)pr.conv[pass][k] : 1e9 + (double)kernel_rank(k);
        };
        auto usable = [&](int pass, int k) { return ws_of(pass, k) != kNoKernel && (!is_winograd(k) || n.winograd == 1 || (n.winograd == 2 && winograd_tile(k) == 2)); };
        const bool need_dx = buf_of(n, l.inputs[0]) >= 0;
        if (n.pinned_kernels[i] >= 0) {  // the caller named the kernels: the layer's only way to run
            const int kf = n.pinned_kernels[i] & 15, kd = (n.pinned_kernels[i] >> 4) & 15, kb = (n.pinned_kernels[i] >> 8) & 15;
            KernelOption f, b;
            f.fwd = kf; f.ws = ws_of(kPassFwd, kf); f.cost = cost_of(kPassFwd, kf);
            b.bd = need_dx ? kd : kKernelGather; b.bf = kb;
            b.ws = std::max(ws_of(kPassBwdFilter, kb), need_dx ? ws_of(kPassBwdData, kd) : (size_t)0);
            b.cost = cost_of(kPassBwdFilter, kb) + (need_dx ? cost_of(kPassBwdData, kd) : 0.0);
            n.options_fwd[i].push_back(f);
            n.options_bwd[i].push_back(b);
            continue;
        }
        for (int k = 0; k < kNumKernels; ++k) {
            if (!usable(kPassFwd, k)) continue;
            KernelOption o;
            o.fwd = k; o.ws = ws_of(kPassFwd, k); o.cost = cost_of(kPassFwd, k);
            n.options_fwd[i].push_back(o);
        }
        for (int kf = 0; kf < kNumKernels; ++kf) {
            if (!usable(kPassBwdFilter, kf)) continue;
            for (int kd = 0; kd < kNumKernels; ++kd) {
                if (need_dx ? !usable(kPassBwdData, kd) : kd != kKernelGather) continue;
                KernelOption o;
                o.bf = kf; o.bd = kd;
                o.ws = std::max(ws_of(kPassBwdFilter, kf), need_dx ? ws_of(kPassBwdData, kd) : (size_t)0);
                o.cost = cost_of(kPassBwdFilter, kf) + (need_dx ? cost_of(kPassBwdData, kd) : 0.0);
                n.options_bwd[i].push_back(o);
            }
        }
        sort_and_prune(n.options_fwd[i]);
        sort_and_prune(n.options_bwd[i]);
        // the last option is always the memory-optimal algorithm: gather kernels, no workspace
    }
}

bool selected(const vdnn_net& n, int b, int policy) {
    const Buffer& B = n.B(b);
    if (B.bwd_users.empty()) return false;
    bool conv = false, pool = false;
    for (int r : B.readers) {
        const int t = n.layers[r].type;
        conv |= t == VDNN_CONV;
        pool |= t == VDNN_MAXPOOL || t == VDNN_AVGPOOL;
    }
    if (policy == VDNN_POLICY_ALL) return conv || pool;
    if (policy == VDNN_POLICY_CONV) return conv;
    return false;
}

size_t baseline_bytes(const vdnn_net& n) {
    const int L = (int)n.layers.size();
    size_t fm = 0, wb = 0, gmax = 0, wmax = 0;
    for (int b = -1; b < L; ++b) {
        const size_t s = n.B(b).count ? align_up(n.B(b).count * 4) : 0;
        fm += s;
        if (b >= 0) gmax = std::max(gmax, s);
    }
    for (int i = 0; i < L; ++i) {
        if (n.layers[i].wcount) wb += 2 * align_up(n.layers[i].wcount * 4);
        if (!n.options_fwd[i].empty()) wmax = std::max(wmax, std::max(n.options_fwd[i][0].ws, n.options_bwd[i][0].ws));
    }
    return fm + wb + 2 * gmax + align_up(wmax);
}

}  // namespace vdnn
