// HBM-bound layers: in-place ReLU, max / average pooling, softmax cross-entropy, channel concat,
// gradient accumulation.  One pass over the data each, coalesced along the innermost (W) axis,
// wavefront-level (64 lanes) reductions, no atomics (results are run-to-run identical).
#include "ops.h"

namespace vdnn {

static inline int grid_for(size_t work, int threads) {
    // enough workgroups to fill 256 CUs several times over; kernels grid-stride beyond that
    return (int)std::max<size_t>(1, std::min<size_t>((work + threads - 1) / threads, 256 * 32));
}

// ---- ReLU (Section 2.2 footnote: activations are computed in place; only Y and dY exist) ------
__global__ void relu_fwd_kernel(float* __restrict__ y, size_t count) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t n4 = count / 4;
    float4* y4 = reinterpret_cast<float4*>(y);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        float4 v = y4[i];
        v.x = v.x > 0.f ? v.x : 0.f;
        v.y = v.y > 0.f ? v.y : 0.f;
        v.z = v.z > 0.f ? v.z : 0.f;
        v.w = v.w > 0.f ? v.w : 0.f;
        y4[i] = v;
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) y[i] = y[i] > 0.f ? y[i] : 0.f;
}

__global__ void relu_bwd_kernel(const float* __restrict__ y, float* __restrict__ dy, size_t count) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t n4 = count / 4;
    const float4* y4 = reinterpret_cast<const float4*>(y);
    float4* d4 = reinterpret_cast<float4*>(dy);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        const float4 a = y4[i];
        float4 g = d4[i];
        g.x = a.x > 0.f ? g.x : 0.f;
        g.y = a.y > 0.f ? g.y : 0.f;
        g.z = a.z > 0.f ? g.z : 0.f;
        g.w = a.w > 0.f ? g.w : 0.f;
        d4[i] = g;
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) dy[i] = y[i] > 0.f ? dy[i] : 0.f;
}

hipError_t relu_fwd(float* y, size_t count, hipStream_t st) {
    if (!count) return hipSuccess;
    hipLaunchKernelGGL(relu_fwd_kernel, dim3(grid_for(count / 4 + 1, 256)), dim3(256), 0, st, y, count);
    return hipGetLastError();
}

hipError_t relu_bwd(const float* y, float* dy, size_t count, hipStream_t st) {
    if (!count) return hipSuccess;
    hipLaunchKernelGGL(relu_bwd_kernel, dim3(grid_for(count / 4 + 1, 256)), dim3(256), 0, st, y, dy, count);
    return hipGetLastError();
}

// ---- pooling ---------------------------------------------------------------------------------
__global__ void maxpool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int H, int W, int P, int Q, int k, int stride,
                                   int pad, size_t total) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int q = (int)(i % Q), p = (int)((i / Q) % P);
        const size_t nc = i / ((size_t)P * Q);
        const float* xp = x + nc * (size_t)H * W;
        float best = -INFINITY;
        for (int r = 0; r < k; ++r) {
            const int h = p * stride + r - pad;
            if ((unsigned)h >= (unsigned)H) continue;
            for (int s = 0; s < k; ++s) {
                const int w = q * stride + s - pad;
                if ((unsigned)w >= (unsigned)W) continue;
                const float v = xp[h * W + w];
                if (v > best) best = v;
            }
        }
        y[i] = best;
    }
}

// One thread per dX element: visit every window that contains it, recompute that window's first
// maximum (row-major scan, strict >) and take the window's dY if this element is it.  Windows are
// visited in ascending (p, q), so overlapping windows add up in a fixed order.
__global__ void maxpool_bwd_kernel(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ dx, int H, int W,
                                   int P, int Q, int k, int stride, int pad, size_t total) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int w = (int)(i % W), h = (int)((i / W) % H);
        const size_t nc = i / ((size_t)H * W);
        const float* xp = x + nc * (size_t)H * W;
        const float* gp = dy + nc * (size_t)P * Q;
        const int p_lo = max(0, (h + pad - k + stride) / stride), p_hi = min(P - 1, (h + pad) / stride);
        const int q_lo = max(0, (w + pad - k + stride) / stride), q_hi = min(Q - 1, (w + pad) / stride);
        float acc = 0.f;
        for (int p = p_lo; p <= p_hi; ++p)
            for (int q = q_lo; q <= q_hi; ++q) {
                float best = -INFINITY;
                int bh = -1, bw = -1;
                for (int r = 0; r < k; ++r) {
                    const int hh = p * stride + r - pad;
                    if ((unsigned)hh >= (unsigned)H) continue;
                    for (int s = 0; s < k; ++s) {
                        const int ww = q * stride + s - pad;
                        if ((unsigned)ww >= (unsigned)W) continue;
                        const float v = xp[hh * W + ww];
                        if (v > best) { best = v; bh = hh; bw = ww; }
                    }
                }
                if (bh == h && bw == w) acc += gp[p * Q + q];
            }
        dx[i] = acc;
    }
}

__global__ void avgpool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int H, int W, int P, int Q, int k, int stride,
                                   int pad, size_t total) {
    const float inv = 1.f / (float)(k * k);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int q = (int)(i % Q), p = (int)((i / Q) % P);
        const size_t nc = i / ((size_t)P * Q);
        const float* xp = x + nc * (size_t)H * W;
        float acc = 0.f;
        for (int r = 0; r < k; ++r) {
            const int h = p * stride + r - pad;
            if ((unsigned)h >= (unsigned)H) continue;
            for (int s = 0; s < k; ++s) {
                const int w = q * stride + s - pad;
                if ((unsigned)w >= (unsigned)W) continue;
                acc += xp[h * W + w];
            }
        }
        y[i] = acc * inv;
    }
}

__global__ void avgpool_bwd_kernel(const float* __restrict__ dy, float* __restrict__ dx, int H, int W, int P, int Q, int k, int stride,
                                   int pad, size_t total) {
    const float inv = 1.f / (float)(k * k);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int w = (int)(i % W), h = (int)((i / W) % H);
        const size_t nc = i / ((size_t)H * W);
        const float* gp = dy + nc * (size_t)P * Q;
        const int p_lo = max(0, (h + pad - k + stride) / stride), p_hi = min(P - 1, (h + pad) / stride);
        const int q_lo = max(0, (w + pad - k + stride) / stride), q_hi = min(Q - 1, (w + pad) / stride);
        float acc = 0.f;
        for (int p = p_lo; p <= p_hi; ++p)
            for (int q = q_lo; q <= q_hi; ++q) acc += gp[p * Q + q];
        dx[i] = acc * inv;
    }
}

static bool pool_dims(int H, int W, int k, int stride, int pad, int* P, int* Q) {
    if (k <= 0 || stride <= 0 || pad < 0 || pad >= k) return false;
    *P = (H + 2 * pad - k) / stride + 1;
    *Q = (W + 2 * pad - k) / stride + 1;
    return *P > 0 && *Q > 0;
}

hipError_t maxpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st) {
    int P, Q;
    if (!pool_dims(H, W, k, stride, pad, &P, &Q)) return hipErrorInvalidValue;
    const size_t total = (size_t)N * C * P * Q;
    hipLaunchKernelGGL(maxpool_fwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, x, y, H, W, P, Q, k, stride, pad, total);
    return hipGetLastError();
}

hipError_t maxpool_bwd(const float* x, const float* dy, float* dx, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st) {
    int P, Q;
    if (!pool_dims(H, W, k, stride, pad, &P, &Q)) return hipErrorInvalidValue;
    const size_t total = (size_t)N * C * H * W;
    hipLaunchKernelGGL(maxpool_bwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, x, dy, dx, H, W, P, Q, k, stride, pad, total);
    return hipGetLastError();
}

hipError_t avgpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st) {
    int P, Q;
    if (!pool_dims(H, W, k, stride, pad, &P, &Q)) return hipErrorInvalidValue;
    const size_t total = (size_t)N * C * P * Q;
    hipLaunchKernelGGL(avgpool_fwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, x, y, H, W, P, Q, k, stride, pad, total);
    return hipGetLastError();
}

hipError_t avgpool_bwd(const float* dy, float* dx, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st) {
    int P, Q;
    if (!pool_dims(H, W, k, stride, pad, &P, &Q)) return hipErrorInvalidValue;
    const size_t total = (size_t)N * C * H * W;
    hipLaunchKernelGGL(avgpool_bwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, dy, dx, H, W, P, Q, k, stride, pad, total);
    return hipGetLastError();
}

// ---- softmax cross-entropy -------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One workgroup; each wavefront takes rows wave, wave + nw, ...; the per-wave partial losses are
// added by one thread in wave order, so the result does not depend on scheduling.
__global__ __launch_bounds__(1024) void softmax_ce_fwd_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels,
                                                               float* __restrict__ loss, int N, int classes) {
    __shared__ float part[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    float wloss = 0.f;
    for (int n = wave; n < N; n += nw) {
        const float* row = z + (size_t)n * classes;
        float m = -INFINITY;
        for (int j = lane; j < classes; j += 64) m = fmaxf(m, row[j]);
        m = wave_max(m);
        float s = 0.f;
        for (int j = lane; j < classes; j += 64) s += expf(row[j] - m);
        s = wave_sum(s);
        wloss += m + logf(s) - row[labels[n]];
    }
    if (lane == 0) part[wave] = wloss;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < nw; ++w) t += part[w];
        *loss = t / (float)N;
    }
}

// One wavefront per row: dz = (softmax(z) - onehot) / N.
__global__ __launch_bounds__(256) void softmax_ce_bwd_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels,
                                                              float* __restrict__ dz, int N, int classes) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (n >= N) return;
    const float* row = z + (size_t)n * classes;
    float m = -INFINITY;
    for (int j = lane; j < classes; j += 64) m = fmaxf(m, row[j]);
    m = wave_max(m);
    float s = 0.f;
    for (int j = lane; j < classes; j += 64) s += expf(row[j] - m);
    s = wave_sum(s);
    const float lse = m + logf(s), invn = 1.f / (float)N;
    const int lab = labels[n];
    float* out = dz + (size_t)n * classes;
    for (int j = lane; j < classes; j += 64) out[j] = (expf(row[j] - lse) - (j == lab ? 1.f : 0.f)) * invn;
}

hipError_t softmax_ce_fwd(const float* z, const int32_t* labels, float* loss, int N, int classes, hipStream_t st) {
    if (N <= 0 || classes <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(softmax_ce_fwd_kernel, dim3(1), dim3(1024), 0, st, z, labels, loss, N, classes);
    return hipGetLastError();
}

hipError_t softmax_ce_bwd(const float* z, const int32_t* labels, float* dz, int N, int classes, hipStream_t st) {
    if (N <= 0 || classes <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(softmax_ce_bwd_kernel, dim3((N + 3) / 4), dim3(256), 0, st, z, labels, dz, N, classes);
    return hipGetLastError();
}

// ---- concat / split along channels, gradient accumulation -------------------------------------
__global__ void concat_copy_kernel(const float* __restrict__ src, float* __restrict__ dst, size_t per_src, size_t per_dst, size_t off,
                                   int to_dst, size_t total) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t n = i / per_src, r = i - n * per_src;
        const size_t j = n * per_dst + off + r;
        if (to_dst) dst[j] = src[i];
        else dst[i] = src[j];
    }
}

// to_dst = 1: big[n][c_off + c][hw] = small[n][c][hw]  (src = small, dst = big)
// to_dst = 0: small[n][c][hw] = big[n][c_off + c][hw]  (src = big,   dst = small)
hipError_t concat_copy(const float* src, float* dst, int N, int c_small, int c_big, int c_off, int hw, int to_dst, hipStream_t st) {
    if (c_off < 0 || c_off + c_small > c_big) return hipErrorInvalidValue;
    const size_t total = (size_t)N * c_small * hw;
    if (!total) return hipSuccess;
    hipLaunchKernelGGL(concat_copy_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, src, dst, (size_t)c_small * hw,
                       (size_t)c_big * hw, (size_t)c_off * hw, to_dst, total);
    return hipGetLastError();
}

__global__ void add_kernel(float* __restrict__ acc, const float* __restrict__ src, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) acc[i] += src[i];
}

hipError_t add_inplace(float* acc, const float* src, size_t count, hipStream_t st) {
    if (!count) return hipSuccess;
    hipLaunchKernelGGL(add_kernel, dim3(grid_for(count, 256)), dim3(256), 0, st, acc, src, count);
    return hipGetLastError();
}

}  // namespace vdnn
