// extern "C" wrappers of the single-layer entry points: argument checks and status mapping only.
#include "../../include/vdnn.h"
#include <cstdio>

#include "ops.h"

using namespace vdnn;

static thread_local char g_op_error[256] = "";

static vdnn_status_t st(hipError_t e) {
    if (e == hipSuccess) return VDNN_OK;
    snprintf(g_op_error, sizeof g_op_error, "%s (%s)", hipGetErrorString(e), hipGetErrorName(e));
    (void)hipGetLastError();
    return e == hipErrorInvalidValue ? VDNN_ERR_INVALID_ARG : VDNN_ERR_HIP;
}

extern "C" const char* vdnn_op_last_error(void) { return g_op_error; }

static bool conv_ok(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    return N > 0 && C > 0 && H > 0 && W > 0 && K > 0 && R > 0 && S > 0 && R == S && stride > 0 && pad >= 0 && H + 2 * pad >= R && W + 2 * pad >= S;
}

extern "C" {

void vdnn_op_set_winograd_chunk_bytes(size_t bytes) { conv_set_winograd_chunk_bytes(bytes); }

size_t vdnn_op_conv_fwd_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    if (!conv_ok(N, C, H, W, K, R, S, stride, pad)) return 0;
    return conv_fwd_workspace(N, C, H, W, K, R, S, stride, pad);
}

size_t vdnn_op_conv_bwd_data_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    if (!conv_ok(N, C, H, W, K, R, S, stride, pad)) return 0;
    return conv_bwd_data_workspace(N, C, H, W, K, R, S, stride, pad);
}

size_t vdnn_op_conv_workspace(int pass, int kernel, int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    if (!conv_ok(N, C, H, W, K, R, S, stride, pad) || pass < 0 || pass > 2) return VDNN_NO_KERNEL;
    return conv_workspace(pass, kernel, N, C, H, W, K, R, S, stride, pad);
}

static bool kernel_ok(int kernel) { return kernel >= VDNN_KERNEL_AUTO && kernel <= VDNN_KERNEL_WINOGRAD4_SMALL; }

vdnn_status_t vdnn_op_conv_fwd(const float* x, const float* w, float* y, void* workspace, size_t workspace_bytes, int N, int C,
                               int H, int W, int K, int R, int S, int stride, int pad, int relu, int kernel, void* stream) {
    if (!x || !w || !y || !conv_ok(N, C, H, W, K, R, S, stride, pad) || !kernel_ok(kernel)) return VDNN_ERR_INVALID_ARG;
    return st(conv_fwd(x, w, y, workspace, workspace_bytes, N, C, H, W, K, R, S, stride, pad, relu, kernel, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_conv_bwd_data(const float* dy, const float* w, float* dx, void* workspace, size_t workspace_bytes, int N,
                                    int C, int H, int W, int K, int R, int S, int stride, int pad, const float* relu_mask,
                                    int kernel, void* stream) {
    if (!dy || !w || !dx || !conv_ok(N, C, H, W, K, R, S, stride, pad) || !kernel_ok(kernel)) return VDNN_ERR_INVALID_ARG;
    return st(conv_bwd_data(dy, w, dx, workspace, workspace_bytes, N, C, H, W, K, R, S, stride, pad, relu_mask, kernel, (hipStream_t)stream));
}

size_t vdnn_op_conv_bwd_filter_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    if (!conv_ok(N, C, H, W, K, R, S, stride, pad)) return 0;
    return conv_bwd_filter_workspace(N, C, H, W, K, R, S, stride, pad);
}

vdnn_status_t vdnn_op_conv_bwd_filter(const float* x, const float* dy, float* dw, void* workspace, size_t workspace_bytes,
                                      int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int kernel, void* stream) {
    if (!x || !dy || !dw || !conv_ok(N, C, H, W, K, R, S, stride, pad) || !kernel_ok(kernel)) return VDNN_ERR_INVALID_ARG;
    return st(conv_bwd_filter(x, dy, dw, workspace, workspace_bytes, N, C, H, W, K, R, S, stride, pad, kernel, (hipStream_t)stream));
}

static_assert(VDNN_STATIC_SCRATCH_BYTES == kStaticScratchBytes, "the header states the size of the static buffer");

vdnn_status_t vdnn_op_conv_bwd_filter_static(const float* x, const float* dy, float* dw, int N, int C, int H, int W, int K, int R, int S,
                                             int stride, int pad, int kernel, void* stream) {
    if (!x || !dy || !dw || !conv_ok(N, C, H, W, K, R, S, stride, pad) || !kernel_ok(kernel)) return VDNN_ERR_INVALID_ARG;
    size_t need = 0;
    const hipError_t e = conv_bwd_filter_static(x, dy, dw, N, C, H, W, K, R, S, stride, pad, kernel, (hipStream_t)stream, &need);
    if (e == hipErrorInvalidValue && need > kStaticScratchBytes) {
        snprintf(g_op_error, sizeof g_op_error, "conv_bwd_filter_static: the kernel needs %zu bytes of workspace, the static buffer holds %zu",
                 need, (size_t)kStaticScratchBytes);
        return VDNN_ERR_INVALID_ARG;
    }
    return st(e);
}

size_t vdnn_op_fc_workspace(int N, int I, int O, int which) {
    if (N <= 0 || I <= 0 || O <= 0 || which < 0 || which > 2) return 0;
    return fc_workspace(N, I, O, which);
}

vdnn_status_t vdnn_op_fc_fwd(const float* x, const float* w, float* y, void* workspace, size_t workspace_bytes, int N, int I,
                             int O, void* stream) {
    if (!x || !w || !y || N <= 0 || I <= 0 || O <= 0) return VDNN_ERR_INVALID_ARG;
    return st(fc_fwd(x, w, y, workspace, workspace_bytes, N, I, O, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_fc_bwd_data(const float* dy, const float* w, float* dx, void* workspace, size_t workspace_bytes, int N,
                                  int I, int O, void* stream) {
    if (!dy || !w || !dx || N <= 0 || I <= 0 || O <= 0) return VDNN_ERR_INVALID_ARG;
    return st(fc_bwd_data(dy, w, dx, workspace, workspace_bytes, N, I, O, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_fc_bwd_filter(const float* x, const float* dy, float* dw, void* workspace, size_t workspace_bytes, int N,
                                    int I, int O, void* stream) {
    if (!x || !dy || !dw || N <= 0 || I <= 0 || O <= 0) return VDNN_ERR_INVALID_ARG;
    return st(fc_bwd_filter(x, dy, dw, workspace, workspace_bytes, N, I, O, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_relu_fwd(float* y, size_t count, void* stream) {
    if (!y && count) return VDNN_ERR_INVALID_ARG;
    return st(relu_fwd(y, count, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_relu_bwd(const float* y, float* dy, size_t count, void* stream) {
    if ((!y || !dy) && count) return VDNN_ERR_INVALID_ARG;
    return st(relu_bwd(y, dy, count, (hipStream_t)stream));
}

static bool pool_ok(const void* a, const void* b, int N, int C, int H, int W, int k, int stride, int pad) {
    return a && b && N > 0 && C > 0 && H > 0 && W > 0 && k > 0 && stride > 0 && pad >= 0 && pad < k && H + 2 * pad >= k && W + 2 * pad >= k;
}

vdnn_status_t vdnn_op_maxpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, void* stream) {
    if (!pool_ok(x, y, N, C, H, W, k, stride, pad)) return VDNN_ERR_INVALID_ARG;
    return st(maxpool_fwd(x, y, N, C, H, W, k, stride, pad, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_maxpool_bwd(const float* x, const float* dy, float* dx, int N, int C, int H, int W, int k, int stride,
                                  int pad, int relu_mask, void* stream) {
    if (!dy || !pool_ok(x, dx, N, C, H, W, k, stride, pad)) return VDNN_ERR_INVALID_ARG;
    return st(maxpool_bwd(x, dy, dx, N, C, H, W, k, stride, pad, relu_mask, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_avgpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, void* stream) {
    if (!pool_ok(x, y, N, C, H, W, k, stride, pad)) return VDNN_ERR_INVALID_ARG;
    return st(avgpool_fwd(x, y, N, C, H, W, k, stride, pad, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_avgpool_bwd(const float* dy, float* dx, int N, int C, int H, int W, int k, int stride, int pad, void* stream) {
    if (!pool_ok(dy, dx, N, C, H, W, k, stride, pad)) return VDNN_ERR_INVALID_ARG;
    return st(avgpool_bwd(dy, dx, N, C, H, W, k, stride, pad, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_softmax_ce_fwd(const float* z, const int32_t* labels, float* loss, int N, int classes, void* stream) {
    if (!z || !labels || !loss || N <= 0 || classes <= 0) return VDNN_ERR_INVALID_ARG;
    return st(softmax_ce_fwd(z, labels, loss, nullptr, N, classes, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_softmax_ce_bwd(const float* z, const int32_t* labels, float* dz, int N, int classes, void* stream) {
    if (!z || !labels || !dz || N <= 0 || classes <= 0) return VDNN_ERR_INVALID_ARG;
    return st(softmax_ce_bwd(z, labels, dz, N, classes, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_concat_copy(const float* src, float* dst, int N, int c_small, int c_big, int c_off, int hw, int to_big,
                                  void* stream) {
    if (!src || !dst || N <= 0 || c_small <= 0 || c_big <= 0 || hw <= 0) return VDNN_ERR_INVALID_ARG;
    return st(concat_copy(src, dst, N, c_small, c_big, c_off, hw, to_big, (hipStream_t)stream));
}

vdnn_status_t vdnn_op_add(float* acc, const float* src, size_t count, void* stream) {
    if ((!acc || !src) && count) return VDNN_ERR_INVALID_ARG;
    return st(add_inplace(acc, src, count, (hipStream_t)stream));
}

}  // extern "C"
