// Winograd F(4x4, 3x3): the minimal-filtering form with interpolation points 0, +-1, +-2 and infinity.  Same structure as
// the F(2x2, 3x3) kernels of winograd.h (Y = A^T [ (G g G^T) .* (B^T d B) ] A per output tile, the products summed over
// channels as grouped GEMMs), with 4x4 output tiles cut from 6x6 input patches: 36 products per 16 outputs, 4x fewer
// multiplications than the direct form, and transformed tensors of 2.25x the size of the tensor (F(2x2): 4x).  Tiles that
// hang over the edge of an image read zeros and drop their extra outputs.  The price is rounding: the transforms carry
// factors up to 8 and sixths, and fp32 results sit about ten times further from the exact ones than F(2x2)'s (some 1e-5 of
// the largest value of a tensor).
//
//   B^T = [4  0 -5  0 1 0]   G = [ 1/4    0     0  ]   A^T = [1 1  1 1  1 0]
//         [0 -4 -4  1 1 0]       [-1/6  -1/6  -1/6 ]         [0 1 -1 2 -2 0]
//         [0  4 -4 -1 1 0]       [-1/6   1/6  -1/6 ]         [0 1  1 4  4 0]
//         [0 -2 -1  2 1 0]       [ 1/24  1/12  1/6 ]         [0 1 -1 8 -8 1]
//         [0  2 -1 -2 1 0]       [ 1/24 -1/12  1/6 ]
//         [0  4  0 -5 0 1]       [  0     0     1  ]
//
// Layouts (T = ceil(H/4)*ceil(W/4) tiles per image, nb images per chunk):
//   U [36][Cred][rows]    V [36][nb][Cred][T]    Mt[36][nb][rows][T]
// Backward-filter is the transposed algorithm: dW = G^T [ sum over tiles (A dY_tile A^T) .* (B^T d B) ] G.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vdnn {

__device__ __forceinline__ void w4_bt(float d0, float d1, float d2, float d3, float d4, float d5, float* r) {  // r = B^T d
    r[0] = 4.f * d0 - 5.f * d2 + d4;
    r[1] = (d3 + d4) - 4.f * (d1 + d2);
    r[2] = 4.f * (d1 - d2) + (d4 - d3);
    r[3] = 2.f * (d3 - d1) + (d4 - d2);
    r[4] = 2.f * (d1 - d3) + (d4 - d2);
    r[5] = 4.f * d1 - 5.f * d3 + d5;
}

__device__ __forceinline__ void w4_at(float m0, float m1, float m2, float m3, float m4, float m5, float* s) {  // s = A^T m
    const float a = m1 + m2, b = m1 - m2, c = m3 + m4, d = m3 - m4;
    s[0] = m0 + a + c;
    s[1] = b + 2.f * d;
    s[2] = a + 4.f * c;
    s[3] = b + 8.f * d + m5;
}

__device__ __forceinline__ void w4_a(float y0, float y1, float y2, float y3, float* a) {  // a = A y
    const float e = y0 + y2, o = y1 + y3, e4 = y0 + 4.f * y2, o4 = 2.f * y1 + 8.f * y3;
    a[0] = y0;
    a[1] = e + o;
    a[2] = e - o;
    a[3] = e4 + o4;
    a[4] = e4 - o4;
    a[5] = y3;
}

__device__ __forceinline__ void w4_g(float g0, float g1, float g2, float* u) {  // u = G g
    const float s = g0 + g2;
    u[0] = 0.25f * g0;
    u[1] = (-1.f / 6.f) * (s + g1);
    u[2] = (-1.f / 6.f) * (s - g1);
    u[3] = (1.f / 24.f) * g0 + (1.f / 12.f) * g1 + (1.f / 6.f) * g2;
    u[4] = (1.f / 24.f) * g0 - (1.f / 12.f) * g1 + (1.f / 6.f) * g2;
    u[5] = g2;
}

__device__ __forceinline__ void w4_gt(float u0, float u1, float u2, float u3, float u4, float u5, float* g) {  // g = G^T u
    g[0] = 0.25f * u0 - (1.f / 6.f) * (u1 + u2) + (1.f / 24.f) * (u3 + u4);
    g[1] = (1.f / 6.f) * (u2 - u1) + (1.f / 12.f) * (u3 - u4);
    g[2] = (1.f / 6.f) * ((u3 + u4) - (u1 + u2)) + u5;
}

// U[xi][cred][row] = (G g G^T)[xi]; g as in wino_filter_kernel (backward-data: W[cred][row] with both taps flipped).
__global__ void wino4_filter_kernel(const float* __restrict__ w, float* __restrict__ u, int K, int C, int bwd) {
    const int rows = bwd ? C : K, cred = bwd ? K : C;
    const size_t total = (size_t)rows * cred;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int row = (int)(i % rows), cr = (int)(i / rows);
        const float* g = bwd ? w + ((size_t)cr * C + row) * 9 : w + ((size_t)row * C + cr) * 9;
        float f[3][3];
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int b = 0; b < 3; ++b) f[a][b] = bwd ? g[(2 - a) * 3 + (2 - b)] : g[a * 3 + b];
        float t[3][6];  // t[b][.] = G applied down column b
#pragma unroll
        for (int b = 0; b < 3; ++b) w4_g(f[0][b], f[1][b], f[2][b], t[b]);
#pragma unroll
        for (int a = 0; a < 6; ++a) {
            float o[6];
            w4_g(t[0][a], t[1][a], t[2][a], o);
#pragma unroll
            for (int b = 0; b < 6; ++b) u[((size_t)(a * 6 + b) * cred + cr) * rows + row] = o[b];
        }
    }
}

// V[xi][n][c][t] = (B^T d B)[xi], d = the 6x6 patch of src[n0 + n][c] whose top-left corner is (4*ty - 1, 4*tx - 1).
// One workgroup stages `pl` consecutive channel planes of an image with their zero borders in LDS (rows of 4 ceil(W/4) + 4
// floats, so that every patch row starts on a 16-byte boundary); threads then walk over the pl * T tiles, which are
// consecutive in V as well, so that every store of a wavefront is one contiguous run whatever the plane size.  pl divides
// Cred and is chosen by the launcher: enough tiles for the workgroup's threads, LDS within kWino4PlaneBytesMax.
// grid (Cred / pl, nb); dynamic LDS pl * (4 ceil(H/4) + 2) * (4 ceil(W/4) + 4) floats.
constexpr size_t kWino4PlaneBytesMax = 64 << 10;
__global__ __launch_bounds__(256) void wino4_input_plane_kernel(const float* __restrict__ src, float* __restrict__ v, int n0, int nb, int C, int H,
                                                                 int W, int pl) {
    extern __shared__ __align__(16) float plane4[];
    const int c0 = blockIdx.x * pl, n = blockIdx.y;
    const int TW = (W + 3) >> 2, TH = (H + 3) >> 2, T = TH * TW;
    const int PW = 4 * TW + 4, PH = 4 * TH + 2, PP = PH * PW;
    const int HW = H * W;
    const float* g = src + ((size_t)(n0 + n) * C + c0) * HW;
    for (int i = threadIdx.x; i < (pl * PP) >> 2; i += blockDim.x) reinterpret_cast<float4*>(plane4)[i] = make_float4(0.f, 0.f, 0.f, 0.f);  // PW % 4 == 0
    __syncthreads();
    if ((W & 3) == 0) {  // rows of 16-byte groups: a group never straddles rows or planes
        const int W4 = W >> 2, total4 = (pl * HW) >> 2;
        for (int i = threadIdx.x; i < total4; i += blockDim.x) {
            const float4 e = reinterpret_cast<const float4*>(g)[i];
            const int row = i / W4, w4 = i - row * W4;  // row counts over all planes
            const int p = row / H, ih = row - p * H;
            float* d = plane4 + p * PP + (ih + 1) * PW + 4 * w4 + 1;
            d[0] = e.x, d[1] = e.y, d[2] = e.z, d[3] = e.w;
        }
    } else {
        for (int i = threadIdx.x; i < pl * HW; i += blockDim.x) {
            const int p = i / HW, r = i - p * HW;
            const int ih = r / W, iw = r - ih * W;
            plane4[p * PP + (ih + 1) * PW + iw + 1] = g[i];
        }
    }
    __syncthreads();
    const size_t gstride = (size_t)nb * C * T;
    for (int i = threadIdx.x; i < pl * T; i += blockDim.x) {
        const int p = i / T, t = i - p * T;
        const int ty = t / TW, tx = t - ty * TW;
        const float* p0 = plane4 + p * PP + 4 * ty * PW + 4 * tx;
        float r[6][6];  // r[j][.] = B^T applied down column j
        float d[6][6];
#pragma unroll
        for (int a = 0; a < 6; ++a) {
            const float4 lo = *reinterpret_cast<const float4*>(p0 + a * PW);
            const float2 hi = *reinterpret_cast<const float2*>(p0 + a * PW + 4);
            d[a][0] = lo.x, d[a][1] = lo.y, d[a][2] = lo.z, d[a][3] = lo.w, d[a][4] = hi.x, d[a][5] = hi.y;
        }
#pragma unroll
        for (int j = 0; j < 6; ++j) w4_bt(d[0][j], d[1][j], d[2][j], d[3][j], d[4][j], d[5][j], r[j]);
        float* o = v + ((size_t)n * C + c0) * T + i;  // planes c0 .. c0 + pl - 1 follow one another in V
#pragma unroll
        for (int a = 0; a < 6; ++a) {
            float q[6];
            w4_bt(r[0][a], r[1][a], r[2][a], r[3][a], r[4][a], r[5][a], q);
#pragma unroll
            for (int j = 0; j < 6; ++j) o[(size_t)(a * 6 + j) * gstride] = q[j];
        }
    }
}

// The same transform for larger planes, read from memory with bounds checks.  grid (ceil(T / blockDim.x), Cred, nb).
__global__ void wino4_input_kernel(const float* __restrict__ src, float* __restrict__ v, int n0, int nb, int C, int H, int W) {
    const int TW = (W + 3) >> 2, T = ((H + 3) >> 2) * TW;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const int c = blockIdx.y, n = blockIdx.z;
    const int ty = t / TW, tx = t - ty * TW;
    const float* plane = src + ((size_t)(n0 + n) * C + c) * H * W;
    float r[6][6];
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        const int iw = 4 * tx - 1 + j;
        float d[6];
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            const int ih = 4 * ty - 1 + i;
            d[i] = ((unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W) ? plane[ih * W + iw] : 0.f;
        }
        w4_bt(d[0], d[1], d[2], d[3], d[4], d[5], r[j]);
    }
    const size_t gstride = (size_t)nb * C * T;
    float* o = v + ((size_t)n * C + c) * T + t;
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        float q[6];
        w4_bt(r[0][i], r[1][i], r[2][i], r[3][i], r[4][i], r[5][i], q);
#pragma unroll
        for (int j = 0; j < 6; ++j) o[(size_t)(i * 6 + j) * gstride] = q[j];
    }
}

// out[n0 + n][row][4ty + i][4tx + j] = (A^T m A)[i][j], m[xi] = Mt[xi][n][row][t]; ReLU / mask as in wino_output_kernel.
// grid (ceil(rows * T / blockDim.x), nb).
__global__ __launch_bounds__(256) void wino4_output_kernel(const float* __restrict__ mt, float* __restrict__ out, const float* __restrict__ mask,
                                                            int n0, int nb, int rows, int H, int W, int relu) {
    const int TW = (W + 3) >> 2, T = ((H + 3) >> 2) * TW;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * T) return;
    const int row = idx / T, t = idx - row * T, n = blockIdx.y;
    const int ty = t / TW, tx = t - ty * TW;
    const size_t gstride = (size_t)nb * rows * T;
    const float* mi = mt + ((size_t)n * rows + row) * T + t;
    float s[6][4];  // s[j][.] = A^T applied down column j
#pragma unroll
    for (int j = 0; j < 6; ++j)
        w4_at(mi[(size_t)(0 * 6 + j) * gstride], mi[(size_t)(1 * 6 + j) * gstride], mi[(size_t)(2 * 6 + j) * gstride],
              mi[(size_t)(3 * 6 + j) * gstride], mi[(size_t)(4 * 6 + j) * gstride], mi[(size_t)(5 * 6 + j) * gstride], s[j]);
    const size_t base = (((size_t)(n0 + n) * rows + row) * H + 4 * ty) * W + 4 * tx;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (4 * ty + i >= H) break;
        float y[4];
        w4_at(s[0][i], s[1][i], s[2][i], s[3][i], s[4][i], s[5][i], y);
        if (relu) {
#pragma unroll
            for (int j = 0; j < 4; ++j) y[j] = y[j] > 0.f ? y[j] : 0.f;
        }
        const size_t at = base + (size_t)i * W;
        if ((W & 3) == 0) {  // rows of the tile start on 16-byte boundaries and lie inside the image
            if (mask) {
                const float4 mk = *reinterpret_cast<const float4*>(mask + at);
                if (!(mk.x > 0.f)) y[0] = 0.f;
                if (!(mk.y > 0.f)) y[1] = 0.f;
                if (!(mk.z > 0.f)) y[2] = 0.f;
                if (!(mk.w > 0.f)) y[3] = 0.f;
            }
            *reinterpret_cast<float4*>(out + at) = make_float4(y[0], y[1], y[2], y[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (4 * tx + j >= W) break;
                float val = y[j];
                if (mask && !(mask[at + j] > 0.f)) val = 0.f;
                out[at + j] = val;
            }
        }
    }
}

// Dt[xi][n][k][t] = (A dy A^T)[xi], dy the 4x4 tile (ty, tx) of dY[n0 + n][k] (zeros beyond the edge).
// grid (ceil(K * T / blockDim.x), nb).
__global__ __launch_bounds__(256) void wino4_dy_kernel(const float* __restrict__ dy, float* __restrict__ dt, int n0, int nb, int K, int H, int W) {
    const int TW = (W + 3) >> 2, T = ((H + 3) >> 2) * TW;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= K * T) return;
    const int k = idx / T, t = idx - k * T, n = blockIdx.y;
    const int ty = t / TW, tx = t - ty * TW;
    const float* plane = dy + (((size_t)(n0 + n) * K + k) * H + 4 * ty) * W + 4 * tx;
    float y[4][4];
    if (((W | H) & 3) == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 e = *reinterpret_cast<const float4*>(plane + (size_t)i * W);
            y[i][0] = e.x, y[i][1] = e.y, y[i][2] = e.z, y[i][3] = e.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) y[i][j] = (4 * ty + i < H && 4 * tx + j < W) ? plane[(size_t)i * W + j] : 0.f;
    }
    float a[4][6];  // a[j][.] = A applied down column j
#pragma unroll
    for (int j = 0; j < 4; ++j) w4_a(y[0][j], y[1][j], y[2][j], y[3][j], a[j]);
    const size_t gstride = (size_t)nb * K * T;
    float* o = dt + ((size_t)n * K + k) * T + t;
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        float q[6];
        w4_a(a[0][i], a[1][i], a[2][i], a[3][i], q);
#pragma unroll
        for (int j = 0; j < 6; ++j) o[(size_t)(i * 6 + j) * gstride] = q[j];
    }
}

// dW[k][c][3][3] = G^T dU G with dU[xi] = acc[xi][k][c].
__global__ void wino4_filter_grad_kernel(const float* __restrict__ acc, float* __restrict__ dw, size_t kc) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < kc; i += (size_t)gridDim.x * blockDim.x) {
        float r[6][3];  // r[b][.] = G^T applied down column b
#pragma unroll
        for (int b = 0; b < 6; ++b)
            w4_gt(acc[(size_t)(0 * 6 + b) * kc + i], acc[(size_t)(1 * 6 + b) * kc + i], acc[(size_t)(2 * 6 + b) * kc + i],
                  acc[(size_t)(3 * 6 + b) * kc + i], acc[(size_t)(4 * 6 + b) * kc + i], acc[(size_t)(5 * 6 + b) * kc + i], r[b]);
        float* o = dw + i * 9;
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            float q[3];
            w4_gt(r[0][a], r[1][a], r[2][a], r[3][a], r[4][a], r[5][a], q);
            o[a * 3 + 0] = q[0], o[a * 3 + 1] = q[1], o[a * 3 + 2] = q[2];
        }
    }
}

}  // namespace vdnn
