// Winograd F(2x2, 3x3) convolution (Lavin & Gray's minimal-filtering form) for 3x3, stride 1, pad 1 layers (an odd
// H or W is covered by tiles that hang over the edge: their extra inputs are zeros, their extra outputs are dropped): Y = A^T [ (G g G^T) .* (B^T d B) ] A per 2x2 output tile, d the 4x4 input patch.  The 16 element-wise
// products, summed over channels, are 16 independent GEMMs [rows x Cred] x [Cred x tiles] that run as one grouped
// launch of conv_fast_kernel (a 1x1 convolution per group); 2.25x fewer multiplications than the direct form.
// This is the kind of performance-optimal algorithm that pays with workspace (Section 2.2 of the paper): the
// transformed filter U, the transformed input V and the products Mt live there, V and Mt for a chunk of images
// at a time so that the workspace stays bounded.
//
// Layouts (T = ceil(H/2)*ceil(W/2) tiles per image, nb images per chunk):
//   U [16][Cred][rows]      rows = output channels of the pass (K forward, C backward-data)
//   V [16][nb][Cred][T]
//   Mt[16][nb][rows][T]
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vdnn {

// U[xi][cred][row] = (G g G^T)[xi] of the 3x3 filter g that pass `bwd` applies for (row, cred):
// forward g = W[row][cred][.][.]; backward-data g = W[cred][row] with both taps flipped.
__global__ void wino_filter_kernel(const float* __restrict__ w, float* __restrict__ u, int K, int C, int bwd) {
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
        float t[4][3];  // G f
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            t[0][b] = f[0][b];
            t[1][b] = 0.5f * (f[0][b] + f[1][b] + f[2][b]);
            t[2][b] = 0.5f * (f[0][b] - f[1][b] + f[2][b]);
            t[3][b] = f[2][b];
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const float o0 = t[a][0], o1 = 0.5f * (t[a][0] + t[a][1] + t[a][2]), o2 = 0.5f * (t[a][0] - t[a][1] + t[a][2]), o3 = t[a][2];
            u[((size_t)(a * 4 + 0) * cred + cr) * rows + row] = o0;
            u[((size_t)(a * 4 + 1) * cred + cr) * rows + row] = o1;
            u[((size_t)(a * 4 + 2) * cred + cr) * rows + row] = o2;
            u[((size_t)(a * 4 + 3) * cred + cr) * rows + row] = o3;
        }
    }
}

// V[xi][n][c][t] = (B^T d B)[xi], d = the 4x4 patch of src[n0 + n][c] whose top-left corner is (2*ty - 1, 2*tx - 1).
// grid (ceil(T / blockDim.x), Cred, nb); lanes walk along tiles.
__global__ void wino_input_kernel(const float* __restrict__ src, float* __restrict__ v, int n0, int nb, int C, int H, int W) {
    const int TW = (W + 1) >> 1, T = ((H + 1) >> 1) * TW;
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const int c = blockIdx.y, n = blockIdx.z;
    const int ty = t / TW, tx = t - ty * TW;
    const float* plane = src + ((size_t)(n0 + n) * C + c) * H * W;
    float d[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ih = 2 * ty - 1 + i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int iw = 2 * tx - 1 + j;
            d[i][j] = ((unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W) ? plane[ih * W + iw] : 0.f;
        }
    }
    float r[4][4];  // B^T d
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        r[0][j] = d[0][j] - d[2][j];
        r[1][j] = d[1][j] + d[2][j];
        r[2][j] = d[2][j] - d[1][j];
        r[3][j] = d[1][j] - d[3][j];
    }
    const size_t gstride = (size_t)nb * C * T;
    float* o = v + ((size_t)n * C + c) * T + t;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[(size_t)(i * 4 + 0) * gstride] = r[i][0] - r[i][2];
        o[(size_t)(i * 4 + 1) * gstride] = r[i][1] + r[i][2];
        o[(size_t)(i * 4 + 2) * gstride] = r[i][2] - r[i][1];
        o[(size_t)(i * 4 + 3) * gstride] = r[i][1] - r[i][3];
    }
}

// The same transform for planes of at most kWinoPlaneMax pixels: one workgroup per (c, n) plane stages the plane with
// its zero border in LDS (each input element read from memory once, coalesced) and its threads walk over the tiles.
// grid (Cred, nb); dynamic LDS (2 ceil(H/2) + 2) * (2 ceil(W/2) + 2) floats.
constexpr int kWinoPlaneMax = 4096;
__global__ void wino_input_plane_kernel(const float* __restrict__ src, float* __restrict__ v, int n0, int nb, int C, int H, int W) {
    extern __shared__ __align__(16) float plane[];
    const int c = blockIdx.x, n = blockIdx.y;
    const int TW = (W + 1) >> 1, TH = (H + 1) >> 1, T = TH * TW;
    const int PW = 2 * TW + 2, PH = 2 * TH + 2;  // the plane with its zero border, rounded up to whole tiles
    const float* g = src + ((size_t)(n0 + n) * C + c) * H * W;
    if ((W & 1) == 0) {
        for (int i = threadIdx.x; i < PW; i += blockDim.x) plane[i] = 0.f, plane[(H + 1) * PW + i] = 0.f;
        if (H & 1) for (int i = threadIdx.x; i < PW; i += blockDim.x) plane[(H + 2) * PW + i] = 0.f;
        for (int i = threadIdx.x; i < H; i += blockDim.x) plane[(i + 1) * PW] = 0.f, plane[(i + 1) * PW + W + 1] = 0.f;
        for (int i = threadIdx.x; i < (H * W) >> 1; i += blockDim.x) {  // W is even: pairs never straddle rows
            const float2 e = reinterpret_cast<const float2*>(g)[i];
            const int h = (2 * i) / W, w = 2 * i - h * W;
            plane[(h + 1) * PW + w + 1] = e.x;
            plane[(h + 1) * PW + w + 2] = e.y;
        }
    } else {
        for (int i = threadIdx.x; i < PH * PW; i += blockDim.x) plane[i] = 0.f;
        __syncthreads();
        for (int i = threadIdx.x; i < H * W; i += blockDim.x) {
            const int h = i / W, w = i - h * W;
            plane[(h + 1) * PW + w + 1] = g[i];
        }
    }
    __syncthreads();
    const size_t gstride = (size_t)nb * C * T;
    for (int t = threadIdx.x; t < T; t += blockDim.x) {
        const int ty = t / TW, tx = t - ty * TW;
        const float* p0 = plane + 2 * ty * PW + 2 * tx;
        float r[4][4];  // B^T d
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float d0 = p0[j], d1 = p0[PW + j], d2 = p0[2 * PW + j], d3 = p0[3 * PW + j];
            r[0][j] = d0 - d2;
            r[1][j] = d1 + d2;
            r[2][j] = d2 - d1;
            r[3][j] = d1 - d3;
        }
        float* o = v + ((size_t)n * C + c) * T + t;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[(size_t)(i * 4 + 0) * gstride] = r[i][0] - r[i][2];
            o[(size_t)(i * 4 + 1) * gstride] = r[i][1] + r[i][2];
            o[(size_t)(i * 4 + 2) * gstride] = r[i][2] - r[i][1];
            o[(size_t)(i * 4 + 3) * gstride] = r[i][1] - r[i][3];
        }
    }
}

// out[n0 + n][row][2ty + i][2tx + j] = (A^T m A)[i][j], m[xi] = Mt[xi][n][row][t]; optional ReLU on the value
// (forward) or zeroing where mask is not positive (backward-data with the preceding in-place ReLU folded in).
// grid (ceil(rows * T / blockDim.x), nb): lanes walk along (row, tile), which is contiguous in Mt.
__global__ void wino_output_kernel(const float* __restrict__ mt, float* __restrict__ out, const float* __restrict__ mask, int n0, int nb,
                                   int rows, int H, int W, int relu) {
    const int TW = (W + 1) >> 1, T = ((H + 1) >> 1) * TW;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * T) return;
    const int row = i / T, t = i - row * T, n = blockIdx.y;
    const int ty = t / TW, tx = t - ty * TW;
    const size_t gstride = (size_t)nb * rows * T;
    const float* mi = mt + ((size_t)n * rows + row) * T + t;
    float m[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) m[i][j] = mi[(size_t)(i * 4 + j) * gstride];
    float s[2][4];  // A^T m
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        s[0][j] = m[0][j] + m[1][j] + m[2][j];
        s[1][j] = m[1][j] - m[2][j] - m[3][j];
    }
    const size_t base = (((size_t)(n0 + n) * rows + row) * H + 2 * ty) * W + 2 * tx;  // even when W is even
    const bool right = 2 * tx + 1 < W;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (2 * ty + i >= H) break;
        float y0 = s[i][0] + s[i][1] + s[i][2], y1 = s[i][1] - s[i][2] - s[i][3];
        if (relu) y0 = y0 > 0.f ? y0 : 0.f, y1 = y1 > 0.f ? y1 : 0.f;
        const size_t idx = base + (size_t)i * W;
        if ((W & 1) == 0) {
            if (mask) {
                const float2 mk = *reinterpret_cast<const float2*>(mask + idx);
                if (!(mk.x > 0.f)) y0 = 0.f;
                if (!(mk.y > 0.f)) y1 = 0.f;
            }
            *reinterpret_cast<float2*>(out + idx) = make_float2(y0, y1);
        } else {
            if (mask && !(mask[idx] > 0.f)) y0 = 0.f;
            out[idx] = y0;
            if (right) {
                if (mask && !(mask[idx + 1] > 0.f)) y1 = 0.f;
                out[idx + 1] = y1;
            }
        }
    }
}

// ---- backward-filter: dW = sum over tiles of G^T [ (A dY_tile A^T) .* (B^T d B) ] G ----
// Dt[xi][n][k][t] = (A dy A^T)[xi], dy the 2x2 tile (ty, tx) of dY[n0 + n][k].  grid (ceil(K * T / blockDim.x), nb):
// lanes walk along (k, tile), which is contiguous in Dt.
__global__ void wino_dy_kernel(const float* __restrict__ dy, float* __restrict__ dt, int n0, int nb, int K, int H, int W) {
    const int TW = (W + 1) >> 1, T = ((H + 1) >> 1) * TW;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= K * T) return;
    const int k = i / T, t = i - k * T, n = blockIdx.y;
    const int ty = t / TW, tx = t - ty * TW;
    const float* plane = dy + (((size_t)(n0 + n) * K + k) * H + 2 * ty) * W + 2 * tx;
    float2 r0, r1;
    if (((W | H) & 1) == 0) {  // even offsets, every tile inside the image
        r0 = *reinterpret_cast<const float2*>(plane), r1 = *reinterpret_cast<const float2*>(plane + W);
    } else {
        const bool right = 2 * tx + 1 < W, below = 2 * ty + 1 < H;
        r0 = make_float2(plane[0], right ? plane[1] : 0.f);
        r1 = make_float2(below ? plane[W] : 0.f, below && right ? plane[W + 1] : 0.f);
    }
    // A = [[1,0],[1,1],[1,-1],[0,-1]]: rows of A dy
    const float a[4][2] = {{r0.x, r0.y}, {r0.x + r1.x, r0.y + r1.y}, {r0.x - r1.x, r0.y - r1.y}, {-r1.x, -r1.y}};
    const size_t gstride = (size_t)nb * K * T;
    float* o = dt + ((size_t)n * K + k) * T + t;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[(size_t)(i * 4 + 0) * gstride] = a[i][0];
        o[(size_t)(i * 4 + 1) * gstride] = a[i][0] + a[i][1];
        o[(size_t)(i * 4 + 2) * gstride] = a[i][0] - a[i][1];
        o[(size_t)(i * 4 + 3) * gstride] = -a[i][1];
    }
}

// acc[i] (+)= sum over s of part[group(i)][s][.], s ascending: part is [groups][splits][K*C], acc is [groups][K*C].
__global__ void wino_accum_kernel(const float* __restrict__ part, float* __restrict__ acc, size_t kc, int splits, int groups, int first) {
    const size_t total = (size_t)groups * kc;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t g = i / kc, e = i - g * kc;
        const float* src = part + g * splits * kc + e;
        float v = src[0];
        for (int s = 1; s < splits; ++s) v += src[(size_t)s * kc];
        acc[i] = first ? v : acc[i] + v;
    }
}

// dW[k][c][3][3] = G^T dU G with dU[xi] = acc[xi][k][c].
__global__ void wino_filter_grad_kernel(const float* __restrict__ acc, float* __restrict__ dw, size_t kc) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < kc; i += (size_t)gridDim.x * blockDim.x) {
        float u[4][4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) u[a][b] = acc[(size_t)(a * 4 + b) * kc + i];
        float r[3][4];  // G^T u, G^T = [[1,.5,.5,0],[0,.5,-.5,0],[0,.5,.5,1]]
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            r[0][b] = u[0][b] + 0.5f * (u[1][b] + u[2][b]);
            r[1][b] = 0.5f * (u[1][b] - u[2][b]);
            r[2][b] = 0.5f * (u[1][b] + u[2][b]) + u[3][b];
        }
        float* o = dw + i * 9;
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            o[a * 3 + 0] = r[a][0] + 0.5f * (r[a][1] + r[a][2]);
            o[a * 3 + 1] = 0.5f * (r[a][1] - r[a][2]);
            o[a * 3 + 2] = 0.5f * (r[a][1] + r[a][2]) + r[a][3];
        }
    }
}

}  // namespace vdnn
