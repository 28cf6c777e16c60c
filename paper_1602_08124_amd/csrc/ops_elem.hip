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
    VDNN_LAUNCH(relu_fwd_kernel, dim3(grid_for(count / 4 + 1, 256)), dim3(256), 0, st, y, count);
    return hipGetLastError();
}

hipError_t relu_bwd(const float* y, float* dy, size_t count, hipStream_t st) {
    if (!count) return hipSuccess;
    VDNN_LAUNCH(relu_bwd_kernel, dim3(grid_for(count / 4 + 1, 256)), dim3(256), 0, st, y, dy, count);
    return hipGetLastError();
}

// ---- pooling ---------------------------------------------------------------------------------
// 32-bit index arithmetic with precomputed reciprocals (tensors have fewer than 2^31 elements).
struct FD { uint32_t m, s; };
static FD make_fd(uint32_t d) {
    FD f; uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    f.s = s;
    f.m = (uint32_t)((((1ull << 32) * ((1ull << s) - d)) / d) + 1);
    return f;
}
__device__ __forceinline__ uint32_t fdiv(uint32_t n, FD f) { return (__umulhi(n, f.m) + n) >> f.s; }

__global__ void maxpool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int H, int W, int P, int Q, int k, int stride,
                                   int pad, uint32_t total, FD fq, FD fp) {
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const uint32_t t = fdiv(i, fq), q = i - t * Q;
        const uint32_t nc = fdiv(t, fp), p = t - nc * P;
        const float* xp = x + (size_t)nc * H * W;
        float best = -INFINITY;
        for (int r = 0; r < k; ++r) {
            const int h = (int)p * stride + r - pad;
            if ((unsigned)h >= (unsigned)H) continue;
            for (int s = 0; s < k; ++s) {
                const int w = (int)q * stride + s - pad;
                if ((unsigned)w >= (unsigned)W) continue;
                const float v = xp[h * W + w];
                if (v > best) best = v;
            }
        }
        y[i] = best;
    }
}

// 3x3 windows, stride 1 or 2: one thread per 2x2 block of outputs.  Their four windows lie in a 4x4 (stride 1) or 5x5
// (stride 2) patch of X that the thread loads once (cells outside the image read as -inf): 4 or 6.25 loads per output
// instead of 9, and the decode of the output index once per four outputs.  Windows are scanned in the same order and
// with the same comparison as in maxpool_fwd_kernel, so the values are the same bits.
template <int STRIDE>
__global__ void maxpool3_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int H, int W, int P, int Q, int pad, uint32_t total,
                                    FD fbq, FD fbp, int nbp, int nbq) {
    constexpr int NB = STRIDE + 3;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const uint32_t t = fdiv(i, fbq);
        const int q0 = 2 * (int)(i - t * (uint32_t)nbq);
        const uint32_t nc = fdiv(t, fbp);
        const int p0 = 2 * (int)(t - nc * (uint32_t)nbp);
        const float* xp = x + (size_t)nc * H * W;
        const int h0 = p0 * STRIDE - pad, w0 = q0 * STRIDE - pad;
        float nb[NB][NB];
#pragma unroll
        for (int a = 0; a < NB; ++a) {
            const int hh = h0 + a;
            const bool okh = (unsigned)hh < (unsigned)H;
            const int hc = min(max(hh, 0), H - 1);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int ww = w0 + b;
                const bool ok = okh && (unsigned)ww < (unsigned)W;
                const float v = xp[hc * W + min(max(ww, 0), W - 1)];
                nb[a][b] = ok ? v : -INFINITY;
            }
        }
        float out[2][2];
#pragma unroll
        for (int dp = 0; dp < 2; ++dp)
#pragma unroll
            for (int dq = 0; dq < 2; ++dq) {
                float best = -INFINITY;
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int s = 0; s < 3; ++s) {
                        const float v = nb[dp * STRIDE + r][dq * STRIDE + s];
                        if (v > best) best = v;
                    }
                out[dp][dq] = best;
            }
        float* yp = y + (size_t)nc * P * Q;
#pragma unroll
        for (int dp = 0; dp < 2; ++dp) {
            if (p0 + dp >= P) continue;
            float* row = yp + (size_t)(p0 + dp) * Q + q0;
            if (q0 + 1 < Q && !(Q & 1)) *reinterpret_cast<float2*>(row) = make_float2(out[dp][0], out[dp][1]);  // q0 and Q even: 8-byte aligned
            else {
                row[0] = out[dp][0];
                if (q0 + 1 < Q) row[1] = out[dp][1];
            }
        }
    }
}

// One thread per dX element: visit every window that contains it, recompute that window's first
// maximum (row-major scan, strict >) and take the window's dY if this element is it.  Windows are
// visited in ascending (p, q), so overlapping windows add up in a fixed order.  relu_mask: the
// pooled tensor is the output of an in-place ReLU whose backward is folded in (dX = 0 where X <= 0).
__global__ void maxpool_bwd_kernel(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ dx, int H, int W,
                                   int P, int Q, int k, int stride, int pad, uint32_t total, FD fw, FD fh, int relu_mask) {
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const uint32_t t = fdiv(i, fw);
        const int w = (int)(i - t * W);
        const uint32_t nc = fdiv(t, fh);
        const int h = (int)(t - nc * H);
        const float* xp = x + (size_t)nc * H * W;
        const float* gp = dy + (size_t)nc * P * Q;
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
        if (relu_mask && !(xp[h * W + w] > 0.f)) acc = 0.f;
        dx[i] = acc;
    }
}

// 3x3 windows (stride 1 or 2, any padding below 3): same rule, one thread per 2x2 block of dX.  For stride 2 the
// block is aligned so that its first row and column start a window; then 2x2 windows (4x4 for stride 1) cover
// it, and they all lie in a 5x5 (6x6) neighbourhood of X that the thread loads into registers once (cells
// outside the image read as -inf, which never wins).  Every window's arg-max is found once and credited to the
// block element it falls on: 25 loads and 4 arg-max searches per four outputs instead of per output.
template <int STRIDE>
__global__ void maxpool3_bwd_kernel(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ dx, int H, int W,
                                    int P, int Q, int pad, uint32_t total, FD fbw, FD fbh, int nbh, int nbw, int relu_mask) {
    constexpr int NWIN = 4 / STRIDE;            // window starts per axis that can touch the block
    constexpr int NB = (NWIN - 1) * STRIDE + 3;  // neighbourhood edge: 5 (stride 2) or 6 (stride 1)
    const int shift = STRIDE == 2 ? (pad & 1) : 0;  // block origin = 2 * index - shift: (origin + pad) is a multiple of the stride
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const uint32_t t = fdiv(i, fbw);
        const int w0 = 2 * (int)(i - t * (uint32_t)nbw) - shift;
        const uint32_t nc = fdiv(t, fbh);
        const int h0 = 2 * (int)(t - nc * (uint32_t)nbh) - shift;
        const float* xp = x + (size_t)nc * H * W;
        const float* gp = dy + (size_t)nc * P * Q;
        float nb[NB][NB];  // rows h0 - 2 .., columns w0 - 2 ..
#pragma unroll
        for (int a = 0; a < NB; ++a) {
            const int hh = h0 - 2 + a;
            const bool okh = (unsigned)hh < (unsigned)H;
            const int hc = min(max(hh, 0), H - 1);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int ww = w0 - 2 + b;
                const bool ok = okh && (unsigned)ww < (unsigned)W;
                const float v = xp[hc * W + min(max(ww, 0), W - 1)];
                nb[a][b] = ok ? v : -INFINITY;
            }
        }
        float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
        // window starts (h0 - 2 + a * STRIDE, w0 - 2 + b * STRIDE), ascending = ascending (p, q)
#pragma unroll
        for (int a = 0; a < NWIN; ++a) {
            const int hn = h0 - 2 + a * STRIDE + pad;  // = p * STRIDE
            const int p = hn / STRIDE;
            const bool okp = hn >= 0 && (hn % STRIDE) == 0 && p < P;
#pragma unroll
            for (int b = 0; b < NWIN; ++b) {
                const int wn = w0 - 2 + b * STRIDE + pad;
                const int q = wn / STRIDE;
                const bool okq = wn >= 0 && (wn % STRIDE) == 0 && q < Q;
                float best = -INFINITY;
                int br = -1, bs = -1;
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int s2 = 0; s2 < 3; ++s2) {
                        const float v = nb[a * STRIDE + r][b * STRIDE + s2];
                        if (v > best) { best = v; br = a * STRIDE + r; bs = b * STRIDE + s2; }
                    }
                if (okp && okq && (unsigned)(br - 2) < 2u && (unsigned)(bs - 2) < 2u) {
                    const float g = gp[p * Q + q];
#pragma unroll
                    for (int dh = 0; dh < 2; ++dh)
#pragma unroll
                        for (int dw = 0; dw < 2; ++dw)
                            if (br == 2 + dh && bs == 2 + dw) acc[dh][dw] += g;
                }
            }
        }
#pragma unroll
        for (int dh = 0; dh < 2; ++dh)
#pragma unroll
            for (int dw = 0; dw < 2; ++dw) {
                const int h = h0 + dh, w = w0 + dw;
                if ((unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W) {
                    float v = acc[dh][dw];
                    if (relu_mask && !(nb[2 + dh][2 + dw] > 0.f)) v = 0.f;
                    dx[(size_t)nc * H * W + (size_t)h * W + w] = v;
                }
            }
    }
}

// 2x2 stride 2, no padding, H even, W a multiple of 4: one thread per two adjacent windows, float4
// rows in, float2 out (forward) / float4 rows out (backward).  Same tie rule as the general kernel.
__global__ void maxpool2x2_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int W, int Q2, uint32_t total, FD fq2) {
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const uint32_t row = fdiv(i, fq2), j = i - row * Q2;  // row = (nc*P + p), j = pair index in the row
        const float4 a = *reinterpret_cast<const float4*>(x + (size_t)row * 2 * W + 4 * j);
        const float4 b = *reinterpret_cast<const float4*>(x + (size_t)row * 2 * W + W + 4 * j);
        float m0 = a.x; if (a.y > m0) m0 = a.y; if (b.x > m0) m0 = b.x; if (b.y > m0) m0 = b.y;
        float m1 = a.z; if (a.w > m1) m1 = a.w; if (b.z > m1) m1 = b.z; if (b.w > m1) m1 = b.w;
        *reinterpret_cast<float2*>(y + (size_t)row * (2 * Q2) + 2 * j) = make_float2(m0, m1);
    }
}

__global__ void maxpool2x2_bwd_kernel(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ dx, int W, int Q2,
                                      uint32_t total, FD fq2, int relu_mask) {
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const uint32_t row = fdiv(i, fq2), j = i - row * Q2;
        const size_t o0 = (size_t)row * 2 * W + 4 * j, o1 = o0 + W;
        const float4 a = *reinterpret_cast<const float4*>(x + o0);
        const float4 b = *reinterpret_cast<const float4*>(x + o1);
        const float2 g = *reinterpret_cast<const float2*>(dy + (size_t)row * (2 * Q2) + 2 * j);
        float4 da = make_float4(0.f, 0.f, 0.f, 0.f), db = da;
        {   // window 0: a.x a.y / b.x b.y, first maximum in that order
            float m = a.x; int w = 0;
            if (a.y > m) { m = a.y; w = 1; }
            if (b.x > m) { m = b.x; w = 2; }
            if (b.y > m) { m = b.y; w = 3; }
            const float v = (relu_mask && !(m > 0.f)) ? 0.f : g.x;
            if (w == 0) da.x = v; else if (w == 1) da.y = v; else if (w == 2) db.x = v; else db.y = v;
        }
        {
            float m = a.z; int w = 0;
            if (a.w > m) { m = a.w; w = 1; }
            if (b.z > m) { m = b.z; w = 2; }
            if (b.w > m) { m = b.w; w = 3; }
            const float v = (relu_mask && !(m > 0.f)) ? 0.f : g.y;
            if (w == 0) da.z = v; else if (w == 1) da.w = v; else if (w == 2) db.z = v; else db.w = v;
        }
        *reinterpret_cast<float4*>(dx + o0) = da;
        *reinterpret_cast<float4*>(dx + o1) = db;
    }
}

__global__ void avgpool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int H, int W, int P, int Q, int k, int stride,
                                   int pad, uint32_t total, FD fq, FD fp) {
    const float inv = 1.f / (float)(k * k);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const uint32_t t = fdiv(i, fq), q = i - t * Q;
        const uint32_t nc = fdiv(t, fp), p = t - nc * P;
        const float* xp = x + (size_t)nc * H * W;
        float acc = 0.f;
        for (int r = 0; r < k; ++r) {
            const int h = (int)p * stride + r - pad;
            if ((unsigned)h >= (unsigned)H) continue;
            for (int s = 0; s < k; ++s) {
                const int w = (int)q * stride + s - pad;
                if ((unsigned)w >= (unsigned)W) continue;
                acc += xp[h * W + w];
            }
        }
        y[i] = acc * inv;
    }
}

__global__ void avgpool_bwd_kernel(const float* __restrict__ dy, float* __restrict__ dx, int H, int W, int P, int Q, int k, int stride,
                                   int pad, uint32_t total, FD fw, FD fh) {
    const float inv = 1.f / (float)(k * k);
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        const uint32_t t = fdiv(i, fw);
        const int w = (int)(i - t * W);
        const uint32_t nc = fdiv(t, fh);
        const int h = (int)(t - nc * H);
        const float* gp = dy + (size_t)nc * P * Q;
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

static bool small_enough(size_t a, size_t b) { return a < 0x7fffffffULL && b < 0x7fffffffULL; }

hipError_t maxpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st) {
    int P, Q;
    if (!pool_dims(H, W, k, stride, pad, &P, &Q)) return hipErrorInvalidValue;
    const size_t total = (size_t)N * C * P * Q;
    if (!small_enough(total, (size_t)N * C * H * W)) return hipErrorInvalidValue;
    if (k == 2 && stride == 2 && pad == 0 && H % 2 == 0 && W % 4 == 0) {
        const uint32_t t2 = (uint32_t)(total / 2);
        VDNN_LAUNCH(maxpool2x2_fwd_kernel, dim3(grid_for(t2, 256)), dim3(256), 0, st, x, y, W, Q / 2, t2, make_fd(Q / 2));
        return hipGetLastError();
    }
    if (k == 3 && (stride == 1 || stride == 2)) {
        const int nbp = (P + 1) / 2, nbq = (Q + 1) / 2;  // 2x2 blocks of Y per plane
        const size_t blocks = (size_t)N * C * nbp * nbq;
        if (stride == 1)
            VDNN_LAUNCH(maxpool3_fwd_kernel<1>, dim3(grid_for(blocks, 256)), dim3(256), 0, st, x, y, H, W, P, Q, pad, (uint32_t)blocks,
                        make_fd(nbq), make_fd(nbp), nbp, nbq);
        else
            VDNN_LAUNCH(maxpool3_fwd_kernel<2>, dim3(grid_for(blocks, 256)), dim3(256), 0, st, x, y, H, W, P, Q, pad, (uint32_t)blocks,
                        make_fd(nbq), make_fd(nbp), nbp, nbq);
        return hipGetLastError();
    }
    VDNN_LAUNCH(maxpool_fwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, x, y, H, W, P, Q, k, stride, pad,
                       (uint32_t)total, make_fd(Q), make_fd(P));
    return hipGetLastError();
}

hipError_t maxpool_bwd(const float* x, const float* dy, float* dx, int N, int C, int H, int W, int k, int stride, int pad,
                       int relu_mask, hipStream_t st) {
    int P, Q;
    if (!pool_dims(H, W, k, stride, pad, &P, &Q)) return hipErrorInvalidValue;
    const size_t total = (size_t)N * C * H * W;
    if (!small_enough(total, total)) return hipErrorInvalidValue;
    if (k == 2 && stride == 2 && pad == 0 && H % 2 == 0 && W % 4 == 0) {
        const uint32_t t2 = (uint32_t)((size_t)N * C * P * Q / 2);
        VDNN_LAUNCH(maxpool2x2_bwd_kernel, dim3(grid_for(t2, 256)), dim3(256), 0, st, x, dy, dx, W, Q / 2, t2, make_fd(Q / 2), relu_mask);
        return hipGetLastError();
    }
    if (k == 3 && (stride == 1 || stride == 2)) {
        const int shift = stride == 2 ? (pad & 1) : 0;
        const int nbh = (H - 1 + shift) / 2 + 1, nbw = (W - 1 + shift) / 2 + 1;  // 2x2 blocks of dX per plane
        const size_t blocks = (size_t)N * C * nbh * nbw;
        if (stride == 1)
            VDNN_LAUNCH(maxpool3_bwd_kernel<1>, dim3(grid_for(blocks, 256)), dim3(256), 0, st, x, dy, dx, H, W, P, Q, pad, (uint32_t)blocks,
                        make_fd(nbw), make_fd(nbh), nbh, nbw, relu_mask);
        else
            VDNN_LAUNCH(maxpool3_bwd_kernel<2>, dim3(grid_for(blocks, 256)), dim3(256), 0, st, x, dy, dx, H, W, P, Q, pad, (uint32_t)blocks,
                        make_fd(nbw), make_fd(nbh), nbh, nbw, relu_mask);
        return hipGetLastError();
    }
    VDNN_LAUNCH(maxpool_bwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, x, dy, dx, H, W, P, Q, k, stride, pad,
                       (uint32_t)total, make_fd(W), make_fd(H), relu_mask);
    return hipGetLastError();
}

hipError_t avgpool_fwd(const float* x, float* y, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st) {
    int P, Q;
    if (!pool_dims(H, W, k, stride, pad, &P, &Q)) return hipErrorInvalidValue;
    const size_t total = (size_t)N * C * P * Q;
    if (!small_enough(total, (size_t)N * C * H * W)) return hipErrorInvalidValue;
    VDNN_LAUNCH(avgpool_fwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, x, y, H, W, P, Q, k, stride, pad,
                       (uint32_t)total, make_fd(Q), make_fd(P));
    return hipGetLastError();
}

hipError_t avgpool_bwd(const float* dy, float* dx, int N, int C, int H, int W, int k, int stride, int pad, hipStream_t st) {
    int P, Q;
    if (!pool_dims(H, W, k, stride, pad, &P, &Q)) return hipErrorInvalidValue;
    const size_t total = (size_t)N * C * H * W;
    if (!small_enough(total, total)) return hipErrorInvalidValue;
    VDNN_LAUNCH(avgpool_bwd_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, dy, dx, H, W, P, Q, k, stride, pad,
                       (uint32_t)total, make_fd(W), make_fd(H));
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
// A label outside [0, classes) reads nothing: its row contributes NaN to the loss, and the number of such rows goes
// to *bad when the caller gave a place for it.
__global__ __launch_bounds__(1024) void softmax_ce_fwd_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels,
                                                               float* __restrict__ loss, int32_t* __restrict__ bad, int N, int classes) {
    __shared__ float part[16];
    __shared__ int nbad[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    float wloss = 0.f;
    int wbad = 0;
    for (int n = wave; n < N; n += nw) {
        const float* row = z + (size_t)n * classes;
        float m = -INFINITY;
        for (int j = lane; j < classes; j += 64) m = fmaxf(m, row[j]);
        m = wave_max(m);
        float s = 0.f;
        for (int j = lane; j < classes; j += 64) s += expf(row[j] - m);
        s = wave_sum(s);
        const int lab = labels[n];
        const bool ok = lab >= 0 && lab < classes;
        wbad += !ok;
        wloss += m + logf(s) - (ok ? row[lab] : NAN);
    }
    if (lane == 0) { part[wave] = wloss; nbad[wave] = wbad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        int b = 0;
        for (int w = 0; w < nw; ++w) { t += part[w]; b += nbad[w]; }
        *loss = t / (float)N;
        if (bad) *bad = b;
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

hipError_t softmax_ce_fwd(const float* z, const int32_t* labels, float* loss, int32_t* bad_labels, int N, int classes, hipStream_t st) {
    if (N <= 0 || classes <= 0) return hipErrorInvalidValue;
    VDNN_LAUNCH(softmax_ce_fwd_kernel, dim3(1), dim3(1024), 0, st, z, labels, loss, bad_labels, N, classes);
    return hipGetLastError();
}

hipError_t softmax_ce_bwd(const float* z, const int32_t* labels, float* dz, int N, int classes, hipStream_t st) {
    if (N <= 0 || classes <= 0) return hipErrorInvalidValue;
    VDNN_LAUNCH(softmax_ce_bwd_kernel, dim3((N + 3) / 4), dim3(256), 0, st, z, labels, dz, N, classes);
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
    VDNN_LAUNCH(concat_copy_kernel, dim3(grid_for(total, 256)), dim3(256), 0, st, src, dst, (size_t)c_small * hw,
                       (size_t)c_big * hw, (size_t)c_off * hw, to_dst, total);
    return hipGetLastError();
}

__global__ void add_kernel(float* __restrict__ acc, const float* __restrict__ src, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) acc[i] += src[i];
}

__global__ void sgd_kernel(float* __restrict__ w, const float* __restrict__ dw, float lr, size_t count) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) w[i] -= lr * dw[i];
}

hipError_t sgd_update(float* w, const float* dw, float lr, size_t count, hipStream_t st) {
    if (!count) return hipSuccess;
    VDNN_LAUNCH(sgd_kernel, dim3(grid_for(count, 256)), dim3(256), 0, st, w, dw, lr, count);
    return hipGetLastError();
}

hipError_t add_inplace(float* acc, const float* src, size_t count, hipStream_t st) {
    if (!count) return hipSuccess;
    VDNN_LAUNCH(add_kernel, dim3(grid_for(count, 256)), dim3(256), 0, st, acc, src, count);
    return hipGetLastError();
}

}  // namespace vdnn
