// Internal declarations of the layer kernels' host launchers (all pointers are device pointers,
// all launches are asynchronous on the given stream).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <algorithm>

// hipGetLastError() after a launch reports the last error of ANY earlier runtime call of this thread,
// including calls made by other libraries in the process; clear that state first so that the value
// read after the launch belongs to the launch.
#define VDNN_LAUNCH(...)            \
    do {                            \
        (void)hipGetLastError();    \
        hipLaunchKernelGGL(__VA_ARGS__); \
    } while (0)

namespace vdnn {

int gemm_splits(long long m, long long n, long long kred);
size_t gemm_workspace_bytes(long long m, long long n, long long kred);

// The three convolution kernels (Section 2.2: algorithms that trade workspace for speed) and the three passes of a CONV layer.
// kKernelWinogradSmall: the Winograd kernels on chunks of half as many images (a further halving would be the next step; one is
// what the workloads ask for): a few per cent slower, about half the workspace.
// kKernelWinograd4 / 4Small: F(4x4, 3x3) instead of F(2x2, 3x3): 4x instead of 2.25x fewer multiplications, results about ten
// times further from the exact ones (still some 1e-5 of a tensor's largest value).
enum {
    kKernelAuto = -1, kKernelGather = 0, kKernelPacked = 1, kKernelWinograd = 2, kKernelWinogradSmall = 3, kKernelWinograd4 = 4,
    kKernelWinograd4Small = 5, kNumKernels = 6
};
inline bool is_winograd(int kernel) { return kernel >= kKernelWinograd && kernel <= kKernelWinograd4Small; }
inline bool winograd_small(int kernel) { return kernel == kKernelWinogradSmall || kernel == kKernelWinograd4Small; }
inline int winograd_tile(int kernel) { return kernel >= kKernelWinograd4 ? 4 : 2; }   // side of the output tile
// rank of a kernel before anything has been measured: lower = expected faster
inline int kernel_rank(int kernel) {
    switch (kernel) {
        case kKernelWinograd4: return 1;
        case kKernelWinograd4Small: return 2;
        case kKernelWinograd: return 3;
        case kKernelWinogradSmall: return 4;
        case kKernelPacked: return 5;
        default: return 6;
    }
}
enum { kPassFwd = 0, kPassBwdData = 1, kPassBwdFilter = 2 };
constexpr size_t kNoKernel = (size_t)-1;
// Workspace bytes of `kernel` for `pass` over the shape (0 for the gather kernel); kNoKernel where it does not apply.
size_t conv_workspace(int pass, int kernel, int N, int C, int H, int W, int K, int R, int S, int stride, int pad);

// conv_*_workspace: bytes of the fastest algorithm for the shape (Winograd F(2x2,3x3) on wide 3x3 layers, else the
// packed-weight direct kernel; 0 where only the no-workspace kernel applies).  The launchers take the kernel to run
// (hipErrorInvalidValue where it does not apply or the workspace is too small for it); kKernelAuto runs the fastest
// one that the workspace they are given has room for.
// conv_*_packed_workspace: bytes of the packed-weight direct kernel alone (what a Winograd-sized layer falls back to).
void conv_set_winograd_chunk_bytes(size_t bytes);  // V + Mt bytes per chunk of images (0 = default 384 MiB)
size_t conv_fwd_packed_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
size_t conv_bwd_data_packed_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
size_t conv_bwd_filter_packed_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
size_t conv_fwd_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
size_t conv_bwd_data_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
hipError_t conv_fwd(const float* x, const float* w, float* y, void* ws, size_t ws_bytes, int N, int C, int H, int W, int K, int R,
                    int S, int stride, int pad, int relu, int kernel, hipStream_t st);
// relu_mask (may be null): tensor of dX's shape; dX is zeroed where it is not positive.
hipError_t conv_bwd_data(const float* dy, const float* w, float* dx, void* ws, size_t ws_bytes, int N, int C, int H, int W, int K,
                         int R, int S, int stride, int pad, const float* relu_mask, int kernel, hipStream_t st);
size_t conv_bwd_filter_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
hipError_t conv_bwd_filter(const float* x, const float* dy, float* dw, void* ws, size_t ws_bytes, int N, int C, int H, int W,
                           int K, int R, int S, int stride, int pad, int kernel, hipStream_t st);

// Backward-filter on the library's own static device buffer instead of a caller's workspace; see ops_gemm.hip.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
hipError_t conv_bwd_filter_static(const float* x, const float* dy, float* dw, int N, int C, int H, int W, int K, int R, int S, int stride,
                                  int pad, int kernel, hipStream_t st, size_t* need);

size_t fc_workspace(int N, int I, int O, int which);
hipError_t fc_fwd(const float* x, const float* w, float* y, void* ws, size_t ws_bytes, int N, int I, int O, hipStream_t st);
hipError_t fc_bwd_data(const float* dy, const float* w, float* dx, void* ws, size_t ws_bytes, int N, int I, int O, hipStream_t st);
hipError_t fc_bwd_filter(const float* x, const float* dy, float* dw, void* ws, size_t ws_bytes, int N, int I, int O, hipStream_t st);

hipError_t relu_fwd(float* y, size_t count, hipStream_t st);
hipError_t relu_bwd(const float* y, float* dy, size_t count, hipStream_t st);
hipError_t maxpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st);
hipError_t maxpool_bwd(const float* x, const float* dy, float* dx, int N, int C, int H, int W, int k, int stride, int pad, int relu_mask,
                       hipStream_t st);
hipError_t avgpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st);
hipError_t avgpool_bwd(const float* dy, float* dx, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st);
// bad_labels (may be null): receives the number of labels outside [0, classes); such a row reads nothing and makes the loss NaN
hipError_t softmax_ce_fwd(const float* z, const int32_t* labels, float* loss, int32_t* bad_labels, int N, int classes, hipStream_t st);
hipError_t softmax_ce_bwd(const float* z, const int32_t* labels, float* dz, int N, int classes, hipStream_t st);
hipError_t concat_copy(const float* src, float* dst, int N, int c_src, int c_dst, int c_off, int hw, int to_dst, hipStream_t st);
hipError_t add_inplace(float* acc, const float* src, size_t count, hipStream_t st);
hipError_t sgd_update(float* w, const float* dw, float lr, size_t count, hipStream_t st);

}  // namespace vdnn
