// Launchers for the GEMM-shaped layers: convolution forward / backward-data / backward-filter
// (implicit GEMM on fp32 MFMA, Section 2.2's "memory-optimal" algorithm: X, Y, W only) and the
// three FC products.  Reductions that would leave the chip idle are split across workgroups;
// partial sums go to a caller-provided workspace and are added in a fixed order.
#include <atomic>

#include "conv_fast.h"
#include "winograd.h"
#include "winograd4.h"
#include "gemm_tile.h"
#include "ops.h"

namespace vdnn {

// A kernel that wants more than the default dynamic LDS size has to be told so once.  The entry points are process-wide,
// so the "already done" flag of each kernel instantiation is atomic; two threads that both find it unset both set the same
// attribute value, which is harmless.
static hipError_t allow_smem(std::atomic<bool>& done, const void* kern, size_t smem) {
    if (done.load(std::memory_order_acquire)) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e == hipSuccess) done.store(true, std::memory_order_release);
    return e;
}

// -------------------------------------------------------------------------------------------
// split heuristic (shared by the workspace query and the launch)
// -------------------------------------------------------------------------------------------
static inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

// A split is worth a workgroup from 512 reduction elements on (16 K-steps of 32): with 2048 the 1x1 and late 3x3 layers of
// the GoogLeNet-shaped net, whose reductions are 6 272 ... 100 352 pixels long, filled a tenth of the chip in backward-filter
// (measured with 2048 / 1024 / 512 / 256: GoogLeNet 4744 / 5248 / 5390 / 5264 img/s, AlexNet 14 340 / 15 200 / 15 730 / 15 970).
constexpr int kMinReduction = 512;
int gemm_splits(long long m, long long n, long long kred) {
    const int bm = m <= 64 ? 64 : 128;
    const long long tiles = (long long)cdiv(m, bm) * cdiv(n, 128);
    long long s = std::min<long long>(1024 / tiles, cdiv(kred, kMinReduction));
    return (int)std::max<long long>(1, s);
}

size_t gemm_workspace_bytes(long long m, long long n, long long kred) {
    const int s = gemm_splits(m, n, kred);
    return s > 1 ? (size_t)s * m * n * sizeof(float) : 0;
}

// out[perm(i)] = sum_s ws[s * count + i].  G lanes share an output: lane g adds slices g, g + G, ... in ascending order, then
// the G partial sums are added in ascending g, so the order is fixed (deterministic) for a given shape.  A small output with many
// slices (the 1x1 and narrow layers: 4096 outputs, hundreds of slices) would otherwise run on a handful of workgroups.
// perm: identity (C = 0), or from the backward-filter kernels' [k][tap][c] order to dW's [k][c][tap].
template <int G>
__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ ws, float* __restrict__ out, size_t count, int splits,
                                                            int C, int RS) {
    constexpr int E = 256 / G;  // outputs per workgroup and pass
    __shared__ float part[G][E];
    const int e = threadIdx.x % E, g = threadIdx.x / E;
    for (size_t base = (size_t)blockIdx.x * E; base < count; base += (size_t)gridDim.x * E) {  // the same trip count for the whole workgroup
        const size_t i = base + e;
        float acc = 0.f;
        if (i < count)
            for (int s = g; s < splits; s += G) acc += ws[(size_t)s * count + i];
        if constexpr (G > 1) {
            part[g][e] = acc;
            __syncthreads();
            if (g == 0) {
#pragma unroll
                for (int k = 1; k < G; ++k) acc += part[k][e];
            }
        }
        if (g == 0 && i < count) {
            size_t o = i;
            if (C) {
                const size_t crs = (size_t)C * RS, k = i / crs, r = i - k * crs;
                o = k * crs + (r % C) * RS + r / C;
            }
            out[o] = acc;
        }
        if constexpr (G > 1) __syncthreads();
    }
}

// C, RS: see the kernel (0, 0: no permutation)
static hipError_t launch_reduce(const float* ws, float* out, size_t count, int splits, hipStream_t st, int C = 0, int RS = 0) {
    const int G = (count <= 16384 && splits >= 64) ? 16 : (count <= 131072 && splits >= 16) ? 4 : 1;
    const int blocks = (int)std::min<size_t>((count + 256 / G - 1) / (256 / G), 4096);
    if (G == 16) VDNN_LAUNCH(reduce_splits_kernel<16>, dim3(blocks), dim3(256), 0, st, ws, out, count, splits, C, RS);
    else if (G == 4) VDNN_LAUNCH(reduce_splits_kernel<4>, dim3(blocks), dim3(256), 0, st, ws, out, count, splits, C, RS);
    else VDNN_LAUNCH(reduce_splits_kernel<1>, dim3(blocks), dim3(256), 0, st, ws, out, count, splits, C, RS);
    return hipGetLastError();
}

template <int BM, int BN, int BK, int WM, int WN, int PADA, int PADB, class LA, class LB, class EP>
static hipError_t launch_tile(const typename LA::Params& pa, const typename LB::Params& pb, const EP& ep, int rows, int cols,
                              int ktot, int splits, hipStream_t st) {
    auto kern = gemm_tile_kernel<BM, BN, BK, WM, WN, PADA, PADB, LA, LB, EP>;
    constexpr size_t smem = gemm_smem_bytes<BM, BN, BK, PADA, PADB>();
    static std::atomic<bool> attr_set{false};  // per instantiation
    if (hipError_t e = allow_smem(attr_set, (const void*)kern, smem); e != hipSuccess) return e;
    GridInfo gi;
    gi.tiles_m = cdiv(rows, BM);
    gi.tiles_n = cdiv(cols, BN);
    gi.splits = splits;
    gi.ktot = ktot;
    gi.ksplit = cdiv(cdiv(ktot, splits), BK) * BK;
    const long long nb = (long long)gi.tiles_m * gi.tiles_n * splits;
    if (nb <= 0 || nb > 0x7fffffffLL) return hipErrorInvalidValue;
    VDNN_LAUNCH(kern, dim3((unsigned)nb), dim3(kThreads), smem, st, pa, pb, ep, gi);
    return hipGetLastError();
}

// -------------------------------------------------------------------------------------------
// convolution forward and (stride 1) backward-data
// -------------------------------------------------------------------------------------------
static ConvGeom make_geom(const float* src, int N, int C, int H, int W, int R, int S, int stride, int pad, int P, int Q) {
    ConvGeom g;
    g.src = src;
    g.C = C; g.H = H; g.W = W;
    g.R = R; g.S = S; g.stride = stride; g.pad = pad;
    g.P = P; g.Q = Q;
    g.M = N * P * Q;
    g.Ktot = C * R * S;
    g.fd_pq = make_fastdiv((uint32_t)(P * Q));
    g.fd_q = make_fastdiv((uint32_t)Q);
    g.fd_rs = make_fastdiv((uint32_t)(R * S));
    g.fd_s = make_fastdiv((uint32_t)S);
    return g;
}

template <int BM, int BN, int WM, int WN>
static hipError_t conv_gemm_cfg(const GatherKParams& wa, const ConvGeom& g, const ConvOut& eo, hipStream_t st) {
    constexpr int BK = 16, PADA = 2, PADB = 32;
    return launch_tile<BM, BN, BK, WM, WN, PADA, PADB, GatherK<BM, BK, PADA>, Im2colR<BN, BK, PADB>, ConvOut>(
        wa, g, eo, eo.rows, g.M, g.Ktot, 1, st);
}

static hipError_t conv_gemm(const GatherKParams& wa, const ConvGeom& g, const ConvOut& eo, hipStream_t st) {
    if (eo.rows <= 32) return conv_gemm_cfg<32, 256, 1, 4>(wa, g, eo, st);
    if (eo.rows <= 64) return conv_gemm_cfg<64, 256, 1, 4>(wa, g, eo, st);
    return conv_gemm_cfg<128, 128, 2, 2>(wa, g, eo, st);
}

static bool fits_i32(long long v) { return v >= 0 && v < 0x7fffffffLL; }


// ---- fast path: reduction channels a multiple of 16, tensors below 4 GiB (32-bit buffer offsets) ----
static bool fast_ok(long long src_elems, long long w_elems, int cred, int R, int S) {
    return cred % 16 == 0 && src_elems * 4 < 0xfffffff0LL && w_elems * 4 < 0x7fffffffLL && R == S;
}

// Resident workgroups of the packed-weight kernel on 256 CUs: 4 per CU for the 128x128 tile (40 KB of LDS,
// 128 registers per lane), 3 per CU for the 256-pixel tiles (45-48 KB of LDS).  Workgroups are dispatched in
// rounds of this many; when the last round would be mostly empty, or when there are fewer tiles than this
// altogether, the reduction of those tiles is split across the idle workgroups.
static int conv_slots(int /*rows*/) { return 1024; }  // 4 workgroups per CU for every tile shape (registers: 4 waves per SIMD; LDS: <= 40 KB each)

struct TailSplit {
    int full_tiles, tail_tiles, splits, steps_per_split;
    size_t bytes;
};

static TailSplit conv_tail_split(int rows, long long M, int cred, int RS) {
    const int bm = rows <= 32 ? 32 : (rows <= 64 ? 64 : 128), bn = rows <= 64 ? 256 : 128;
    const long long tiles = (long long)cdiv(rows, bm) * cdiv(M, bn);
    const int steps = cred / 16 * RS;
    const int kConvSlots = conv_slots(rows);
    TailSplit t;
    t.full_tiles = (int)(tiles / kConvSlots * kConvSlots);
    t.tail_tiles = (int)(tiles - t.full_tiles);
    t.splits = 1;
    t.steps_per_split = steps;
    t.bytes = 0;
    // only worth it when the job is a few rounds long: measured on VGG-16, 2 rounds gain 9 %, 8 and 16 rounds nothing
    if (t.tail_tiles > 0 && t.tail_tiles * 10 < kConvSlots * 7 && t.full_tiles < 4 * kConvSlots) {
        int s = std::min(std::min(kConvSlots / t.tail_tiles, 8), steps / 8);
        if (s > 1) {
            t.steps_per_split = cdiv(steps, s);
            t.splits = cdiv(steps, t.steps_per_split);
            t.bytes = (size_t)t.tail_tiles * t.splits * bm * bn * sizeof(float);
        }
    }
    if (t.splits == 1) { t.full_tiles += t.tail_tiles; t.tail_tiles = 0; }
    return t;
}

template <int BM, int BN, int WM, int WN, bool QUAD = false>
static hipError_t conv_fast_cfg(ConvFastParams& p, const TailSplit& ts, float* partial, hipStream_t st) {
    auto kern = conv_fast_kernel<BM, BN, WM, WN, false, QUAD>;
    auto kern_split = conv_fast_kernel<BM, BN, WM, WN, true, QUAD>;
    constexpr size_t smem = sizeof(float) * 2 * 16 * ((BM + kConvFastPad<BN>) + (BN + kConvFastPad<BN>));
    static std::atomic<bool> attr_set{false}, attr_set_split{false};
    if (hipError_t e = allow_smem(attr_set, (const void*)kern, smem); e != hipSuccess) return e;
    if (hipError_t e = allow_smem(attr_set_split, (const void*)kern_split, smem); e != hipSuccess) return e;
    p.tiles_m = cdiv(p.rows, BM);
    p.tiles_n = cdiv(p.M, BN);
    if ((long long)p.tiles_m * p.tiles_n != (long long)ts.full_tiles + ts.tail_tiles) return hipErrorInvalidValue;
    const int total_steps = p.Cred / 16 * p.R * p.S;
    if (ts.full_tiles > 0) {
        p.tile_begin = 0; p.n_tiles = ts.full_tiles; p.splits = 1; p.steps_per_split = total_steps; p.partial = nullptr;
        VDNN_LAUNCH(kern, dim3((unsigned)(ts.full_tiles * p.groups)), dim3(kThreads), smem, st, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (ts.tail_tiles > 0) {
        p.tile_begin = ts.full_tiles; p.n_tiles = ts.tail_tiles; p.splits = ts.splits; p.steps_per_split = ts.steps_per_split;
        p.partial = partial;
        VDNN_LAUNCH(kern_split, dim3((unsigned)(ts.tail_tiles * ts.splits)), dim3(kThreads), smem, st, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        VDNN_LAUNCH((conv_split_fixup_kernel<BM, BN>), dim3((unsigned)ts.tail_tiles * kFixupChunks), dim3(kThreads), 0, st, p);
        return hipGetLastError();
    }
    return hipSuccess;
}

// src: the gathered tensor [N][cred][H][W]; w: original KCRS weights; ws: room for the packed copy of W
// followed by the partial sums of split tiles.
static hipError_t conv_fast(const float* src, const float* w, float* ws, const ConvOut& eo, int N, int cred, int H, int W, int K,
                            int C, int R, int S, int stride, int pad, int P, int Q, int bwd, hipStream_t st) {
    const size_t wcount = (size_t)K * C * R * S;
    const int pblocks = (int)std::min<size_t>((wcount + 255) / 256, 4096);
    VDNN_LAUNCH(pack_weights_kernel, dim3(pblocks), dim3(256), 0, st, w, ws, K, C, R * S, bwd);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    ConvFastParams p;
    p.src = src; p.wp = ws;
    p.src_bytes = (uint32_t)((size_t)N * cred * H * W * 4);
    p.wp_bytes = (uint32_t)(wcount * 4);
    p.rows = eo.rows;
    p.Cred = cred; p.H = H; p.W = W;
    p.R = R; p.S = S; p.stride = stride; p.pad = pad;
    p.P = P; p.Q = Q; p.M = N * P * Q;
    p.fd_pq = make_fastdiv((uint32_t)(P * Q));
    p.fd_q = make_fastdiv((uint32_t)Q);
    p.out = eo;
    const TailSplit ts = conv_tail_split(eo.rows, p.M, cred, R * S);
    float* partial = ws + (wcount + 63) / 64 * 64;
    if (eo.rows <= 32) return conv_fast_cfg<32, 256, 1, 4>(p, ts, partial, st);
    const bool quad = eo.rows % 4 == 0;  // weight rows by 16-byte loads
    if (eo.rows <= 64) return quad ? conv_fast_cfg<64, 256, 1, 4, true>(p, ts, partial, st) : conv_fast_cfg<64, 256, 1, 4>(p, ts, partial, st);
    return quad ? conv_fast_cfg<128, 128, 2, 2, true>(p, ts, partial, st) : conv_fast_cfg<128, 128, 2, 2>(p, ts, partial, st);
}

// -------------------------------------------------------------------------------------------
// Winograd F(2x2, 3x3): see winograd.h.  Eligible: 3x3, stride 1, pad 1, reduction channels a multiple
// of 16 and at least 256, rows a multiple of 4 and at least 128: measured on VGG-16 (256), in TFLOP/s of the direct
// form's operation count, the direct kernel's 137 become 234 at 512 x 512 channels (28 x 28), 212 (14 x 14), 196-205 at
// 256 x 512, 185 at 256 x 256 (56 x 56) and 156 at 256 -> 128; with 128 reduction channels the transforms' HBM
// traffic costs what the saved multiplications gain (131 against 136).
// Workspace: U, then V and Mt for `nb` images, nb the largest count that keeps V + Mt within the chunk size.
// -------------------------------------------------------------------------------------------
// Default 384 MiB, measured on VGG-16 (256) with 512 / 448 / 384 / 320 / 256 MiB: the step without a budget 112.3 / 113.0 / 113.5 /
// 116.6 / 119.8 ms, the step under 12 GiB (fit) 210.0 / 198.0 / 187.5 / 192.2 / 195.9 ms: smaller workspaces leave less to offload.
constexpr size_t kWinoChunkDefaultBytes = (size_t)384 << 20;
static size_t g_wino_chunk_bytes = kWinoChunkDefaultBytes;

void conv_set_winograd_chunk_bytes(size_t bytes) { g_wino_chunk_bytes = bytes ? bytes : kWinoChunkDefaultBytes; }

// m: the output tile's side, 2 (F(2x2, 3x3), winograd.h) or 4 (F(4x4, 3x3), winograd4.h); (m + 2)^2 grouped products.
static inline int wino_tiles(int H, int W, int m) { return cdiv(H, m) * cdiv(W, m); }
static inline int wino_groups(int m) { return (m + 2) * (m + 2); }
// Backward-filter splits the reduction over tile positions so that about 1024 workgroups run (four per compute unit);
// the 36 products of F(4x4) come in counts that fill the last round badly (576 tiles of 128 x 128 for 512 x 512 channels),
// and measured best with up to 2048 (c4_2: 3.18 ms unsplit, 2.74 ms in three splits; c5: 1.03 and 0.91).
static inline int wino_bwdf_max_splits(int K, int C, int m) {
    const long long tiles = (long long)cdiv(K, 128) * (C / 128) * wino_groups(m);
    return (int)std::max<long long>(1, (m == 4 ? 2048 : 1024) / tiles);
}

static bool wino_ok(int N, int cred, int H, int W, int rows, int R, int S, int stride, int pad, int m) {
    return R == 3 && S == 3 && stride == 1 && pad == 1 && cred % 16 == 0 && rows % 4 == 0 && cred >= (m == 4 ? 128 : 256) &&
           rows >= 128 && N >= 1 && cred <= 65535 && rows <= 65535 &&  // the transforms' grids carry channels and images in y and z
           (long long)wino_tiles(H, W, m) <= 32768 &&                  // and index (channel, tile) with 32 bits
           (long long)H * W <= (1 << 24);
}

// Images per chunk: as many as keep the whole workspace within the chunk size (what does not depend on the chunk comes off
// first: the transformed filter; for backward-filter, `bwdf`, the products and the most partial sums a split can take), at
// least one; then evened out over the chunks that this takes (256 images at 167 per chunk run as 128 + 128, not 167 + 89:
// the same number of launches on a smaller workspace).
// small: half as many images per chunk as that, evened out the same way (the _SMALL kernels); equal to the full count
// only where that is one image.
static int wino_chunk(int N, int cred, int H, int W, int rows, int m, bool small = false, bool bwdf = false) {
    const size_t G = (size_t)wino_groups(m);
    const size_t per_image = G * (cred + rows) * wino_tiles(H, W, m) * sizeof(float);
    size_t fixed = (G * cred * rows + 63) / 64 * 64 * sizeof(float);
    if (bwdf) fixed = G * cred * rows * sizeof(float) * (1 + wino_bwdf_max_splits(rows, cred, m));
    const size_t room = g_wino_chunk_bytes > fixed ? g_wino_chunk_bytes - fixed : 0;
    int most = (int)std::max<size_t>(1, std::min<size_t>(std::min<size_t>((size_t)N, 65535), room / per_image));
    int chunks = (N + most - 1) / most;
    if (!small) return (N + chunks - 1) / chunks;
    most = ((N + chunks - 1) / chunks + 1) / 2;
    chunks = (N + most - 1) / most;
    return (N + chunks - 1) / chunks;
}

// V for images [n0, n0 + cur) of src
static hipError_t wino_input(const float* src, float* v, int n0, int cur, int cred, int H, int W, int m, hipStream_t st) {
    const int T = wino_tiles(H, W, m);
    const int tb = T <= 64 ? 64 : 256;
    if (m == 4) {
        const size_t plane_bytes = sizeof(float) * (4 * cdiv(H, 4) + 2) * (4 * cdiv(W, 4) + 4);
        if (plane_bytes <= kWino4PlaneBytesMax && cur <= 65535) {
            // planes per workgroup: enough tiles for a few rounds of its 256 threads, within 32 KB of LDS (cred is a multiple of 16)
            int pl = 1;
            while (pl < 16 && pl * T < 512 && 2 * pl * plane_bytes <= (32 << 10)) pl *= 2;
            VDNN_LAUNCH(wino4_input_plane_kernel, dim3((unsigned)(cred / pl), (unsigned)cur), dim3(256), pl * plane_bytes, st, src, v, n0, cur, cred, H, W, pl);
        } else {
            VDNN_LAUNCH(wino4_input_kernel, dim3((unsigned)cdiv(T, tb), (unsigned)cred, (unsigned)cur), dim3(tb), 0, st, src, v, n0, cur, cred, H, W);
        }
    } else if (H * W <= kWinoPlaneMax && cur <= 65535) {
        VDNN_LAUNCH(wino_input_plane_kernel, dim3((unsigned)cred, (unsigned)cur), dim3(tb), sizeof(float) * (2 * ((H + 1) / 2) + 2) * (2 * ((W + 1) / 2) + 2), st,
                    src, v, n0, cur, cred, H, W);
    } else {
        VDNN_LAUNCH(wino_input_kernel, dim3((unsigned)cdiv(T, tb), (unsigned)cred, (unsigned)cur), dim3(tb), 0, st, src, v, n0, cur, cred, H, W);
    }
    return hipGetLastError();
}

static size_t wino_workspace(int N, int cred, int H, int W, int rows, int m, bool small = false) {
    const int G = wino_groups(m);
    const size_t u = ((size_t)G * cred * rows + 63) / 64 * 64 * sizeof(float);
    return u + (size_t)wino_chunk(N, cred, H, W, rows, m, small) * G * (cred + rows) * wino_tiles(H, W, m) * sizeof(float);
}

// src [N][cred][H][W] -> out [N][rows][H][W]; w is the layer's KCRS filter; bwd selects which way it is applied.
static hipError_t conv_winograd(const float* src, const float* w, float* ws, float* out, const float* mask, int relu, int N, int cred, int H,
                                int W, int rows, int K, int C, int bwd, int m, bool small, hipStream_t st) {
    const int T = wino_tiles(H, W, m), G = wino_groups(m);
    const int nb = wino_chunk(N, cred, H, W, rows, m, small);
    float* u = ws;
    float* v = ws + ((size_t)G * cred * rows + 63) / 64 * 64;
    float* mt = v + (size_t)G * nb * cred * T;
    const size_t wcount = (size_t)rows * cred;
    if (m == 4) VDNN_LAUNCH(wino4_filter_kernel, dim3((unsigned)std::min<size_t>((wcount + 255) / 256, 4096)), dim3(256), 0, st, w, u, K, C, bwd);
    else VDNN_LAUNCH(wino_filter_kernel, dim3((unsigned)std::min<size_t>((wcount + 255) / 256, 4096)), dim3(256), 0, st, w, u, K, C, bwd);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    for (int n0 = 0; n0 < N; n0 += nb) {
        const int cur = std::min(nb, N - n0);
        e = wino_input(src, v, n0, cur, cred, H, W, m, st);
        if (e != hipSuccess) return e;
        ConvFastParams p;
        p.src = v; p.wp = u;
        p.src_bytes = (uint32_t)((size_t)cur * cred * T * 4);
        p.wp_bytes = (uint32_t)((size_t)cred * rows * 4);
        p.rows = rows;
        p.Cred = cred; p.H = cdiv(H, m); p.W = cdiv(W, m);
        p.R = 1; p.S = 1; p.stride = 1; p.pad = 0;
        p.P = cdiv(H, m); p.Q = cdiv(W, m); p.M = cur * T;
        p.fd_pq = make_fastdiv((uint32_t)T);
        p.fd_q = make_fastdiv((uint32_t)cdiv(W, m));
        ConvOut eo;
        eo.out = mt; eo.mask = nullptr; eo.rows = rows; eo.M = p.M; eo.PQ = T; eo.relu = 0; eo.fd_pq = p.fd_pq;
        p.out = eo;
        p.groups = G;
        p.src_gstride = (size_t)cur * cred * T;
        p.wp_gstride = (size_t)cred * rows;
        p.out_gstride = (size_t)cur * rows * T;
        TailSplit ts;
        ts.splits = 1; ts.steps_per_split = cred / 16; ts.bytes = 0; ts.tail_tiles = 0;
        ts.full_tiles = rows <= 64 ? cdiv(p.M, 256) : cdiv(rows, 128) * cdiv(p.M, 128);
        e = rows <= 64 ? conv_fast_cfg<64, 256, 1, 4, true>(p, ts, nullptr, st) : conv_fast_cfg<128, 128, 2, 2, true>(p, ts, nullptr, st);
        if (e != hipSuccess) return e;
        if (m == 4)
            VDNN_LAUNCH(wino4_output_kernel, dim3((unsigned)cdiv(rows * T, 256), (unsigned)cur), dim3(256), 0, st, (const float*)mt, out, mask, n0, cur,
                        rows, H, W, relu);
        else
            VDNN_LAUNCH(wino_output_kernel, dim3((unsigned)cdiv(rows * T, 256), (unsigned)cur), dim3(256), 0, st, (const float*)mt, out, mask, n0, cur,
                        rows, H, W, relu);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

static size_t conv_fast_workspace(size_t wcount, int rows, long long M, int cred, int RS) {
    return (wcount + 63) / 64 * 64 * sizeof(float) + conv_tail_split(rows, M, cred, RS).bytes;
}

// workspace of the packed-weight direct kernel (0: it does not apply)
size_t conv_fwd_packed_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    if (!fast_ok((long long)N * C * H * W, (long long)K * C * R * S, C, R, S)) return 0;
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    return conv_fast_workspace((size_t)K * C * R * S, K, (long long)N * P * Q, C, R * S);
}

size_t conv_bwd_data_packed_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (stride != 1 || pad > R - 1) return 0;
    if (!fast_ok((long long)N * K * P * Q, (long long)K * C * R * S, K, R, S)) return 0;
    return conv_fast_workspace((size_t)K * C * R * S, C, (long long)N * H * W, K, R * S);
}

static bool wino_bwdf_ok(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int m);
static size_t wino_bwdf_workspace(int N, int C, int H, int W, int K, int m, bool small = false);

// Bytes of workspace a kernel needs for a pass over the shape; kNoKernel where that kernel does not apply.
size_t conv_workspace(int pass, int kernel, int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    if (kernel == kKernelGather) return 0;  // works on X, Y and W as stored, for every shape
    if (kernel != kKernelPacked && !is_winograd(kernel)) return kNoKernel;
    const bool small = winograd_small(kernel);
    const int m = winograd_tile(kernel);
    // a small-chunk variant exists where halving the chunk does change it (one image per chunk cannot be halved)
    if (pass == kPassFwd) {
        const size_t packed = conv_fwd_packed_workspace(N, C, H, W, K, R, S, stride, pad);
        if (!packed) return kNoKernel;
        if (kernel == kKernelPacked) return packed;
        if (!wino_ok(N, C, H, W, K, R, S, stride, pad, m) || (small && wino_chunk(N, C, H, W, K, m, true) == wino_chunk(N, C, H, W, K, m))) return kNoKernel;
        return wino_workspace(N, C, H, W, K, m, small);
    }
    if (pass == kPassBwdData) {
        const size_t packed = conv_bwd_data_packed_workspace(N, C, H, W, K, R, S, stride, pad);
        if (!packed) return kNoKernel;
        if (kernel == kKernelPacked) return packed;
        if (!wino_ok(N, K, H, W, C, R, S, stride, pad, m) || (small && wino_chunk(N, K, H, W, C, m, true) == wino_chunk(N, K, H, W, C, m))) return kNoKernel;
        return wino_workspace(N, K, H, W, C, m, small);
    }
    if (pass == kPassBwdFilter) {
        if (is_winograd(kernel)) {
            if (!wino_bwdf_ok(N, C, H, W, K, R, S, stride, pad, m) || (small && wino_chunk(N, C, H, W, K, m, true, true) == wino_chunk(N, C, H, W, K, m, false, true))) return kNoKernel;
            return wino_bwdf_workspace(N, C, H, W, K, m, small);
        }
        const size_t split = conv_bwd_filter_packed_workspace(N, C, H, W, K, R, S, stride, pad);
        return split ? split : kNoKernel;  // no split and no tap-major staging: the same launch as the gather kernel
    }
    return kNoKernel;
}

// The kernels in the order kKernelAuto tries them (the order of kernel_rank).
static constexpr int kAutoOrder[] = {kKernelWinograd4, kKernelWinograd4Small, kKernelWinograd, kKernelWinogradSmall, kKernelPacked};

// workspace of the fastest kernel for the shape and pass (0: only the gather kernel applies)
static size_t fastest_workspace(int pass, int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    for (int k : kAutoOrder) {
        const size_t need = conv_workspace(pass, k, N, C, H, W, K, R, S, stride, pad);
        if (need != kNoKernel) return need;
    }
    return 0;
}

size_t conv_fwd_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    return fastest_workspace(kPassFwd, N, C, H, W, K, R, S, stride, pad);
}

size_t conv_bwd_data_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    return fastest_workspace(kPassBwdData, N, C, H, W, K, R, S, stride, pad);
}

// kernel == kKernelAuto: the fastest kernel whose workspace the caller's has room for.  Otherwise exactly that kernel;
// hipErrorInvalidValue when it does not apply to the shape or the workspace is too small for it.
static int resolve_kernel(int pass, int kernel, const void* ws, size_t ws_bytes, int N, int C, int H, int W, int K, int R, int S, int stride,
                          int pad) {
    if (kernel == kKernelAuto) {
        for (int k : kAutoOrder) {
            const size_t need = conv_workspace(pass, k, N, C, H, W, K, R, S, stride, pad);
            if (need != kNoKernel && ws && ws_bytes >= need) return k;
        }
        return kKernelGather;
    }
    const size_t need = conv_workspace(pass, kernel, N, C, H, W, K, R, S, stride, pad);
    if (need == kNoKernel || (need && (!ws || ws_bytes < need))) return -2;
    return kernel;
}

hipError_t conv_fwd(const float* x, const float* w, float* y, void* ws, size_t ws_bytes, int N, int C, int H, int W, int K, int R, int S, int stride,
                    int pad, int relu, int kernel, hipStream_t st) {
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (P <= 0 || Q <= 0) return hipErrorInvalidValue;
    if (!fits_i32((long long)N * C * H * W) || !fits_i32((long long)N * K * P * Q)) return hipErrorInvalidValue;
    ConvGeom g = make_geom(x, N, C, H, W, R, S, stride, pad, P, Q);
    GatherKParams wa;
    wa.base = w; wa.rows = K; wa.rstride = C * R * S; wa.kstride = 1; wa.rs = 1; wa.flip = 0;
    wa.fd_rs = make_fastdiv(1);
    ConvOut eo;
    eo.out = y; eo.mask = nullptr; eo.rows = K; eo.M = g.M; eo.PQ = P * Q; eo.relu = relu; eo.fd_pq = g.fd_pq;
    const int use = resolve_kernel(kPassFwd, kernel, ws, ws_bytes, N, C, H, W, K, R, S, stride, pad);
    if (use == -2) return hipErrorInvalidValue;
    if (is_winograd(use)) return conv_winograd(x, w, (float*)ws, y, nullptr, relu, N, C, H, W, K, K, C, 0, winograd_tile(use), winograd_small(use), st);
    if (use == kKernelPacked) return conv_fast(x, w, (float*)ws, eo, N, C, H, W, K, C, R, S, stride, pad, P, Q, 0, st);
    return conv_gemm(wa, g, eo, st);
}

// General backward-data for strided convolutions: one thread per dX element, gathers every forward
// term that touched it.  Only first layers are strided in the paper's networks and those need no
// dX, so this path is for completeness, not speed.
__global__ void conv_bwd_data_direct_kernel(const float* __restrict__ dy, const float* __restrict__ w, float* __restrict__ dx,
                                            int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int P, int Q,
                                            const float* __restrict__ relu_mask) {
    const size_t total = (size_t)N * C * H * W;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int wi = (int)(i % W), hi = (int)((i / W) % H), c = (int)((i / ((size_t)W * H)) % C), n = (int)(i / ((size_t)W * H * C));
        float acc = 0.f;
        for (int k = 0; k < K; ++k)
            for (int r = 0; r < R; ++r) {
                const int hn = hi + pad - r;
                if (hn < 0 || hn % stride) continue;
                const int p = hn / stride;
                if (p >= P) continue;
                for (int s = 0; s < S; ++s) {
                    const int wn = wi + pad - s;
                    if (wn < 0 || wn % stride) continue;
                    const int q = wn / stride;
                    if (q >= Q) continue;
                    acc += dy[(((size_t)n * K + k) * P + p) * Q + q] * w[(((size_t)k * C + c) * R + r) * S + s];
                }
            }
        if (relu_mask && !(relu_mask[i] > 0.f)) acc = 0.f;
        dx[i] = acc;
    }
}

hipError_t conv_bwd_data(const float* dy, const float* w, float* dx, void* ws, size_t ws_bytes, int N, int C, int H, int W, int K, int R, int S, int stride,
                         int pad, const float* relu_mask, int kernel, hipStream_t st) {
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (P <= 0 || Q <= 0) return hipErrorInvalidValue;
    if (!fits_i32((long long)N * C * H * W) || !fits_i32((long long)N * K * P * Q)) return hipErrorInvalidValue;
    const int use = resolve_kernel(kPassBwdData, kernel, ws, ws_bytes, N, C, H, W, K, R, S, stride, pad);
    if (use == -2) return hipErrorInvalidValue;
    if (stride != 1 || pad > R - 1 || pad > S - 1) {
        const size_t total = (size_t)N * C * H * W;
        const int blocks = (int)std::min<size_t>((total + 255) / 256, 65535 * 4);
        VDNN_LAUNCH(conv_bwd_data_direct_kernel, dim3(blocks), dim3(256), 0, st, dy, w, dx, N, C, H, W, K, R, S, stride, pad, P, Q, relu_mask);
        return hipGetLastError();
    }
    // dX[n][c][h][w] = sum_{k,r',s'} dY[n][k][h - (R-1-pad) + r'][w - (S-1-pad) + s'] * W[k][c][R-1-r'][S-1-s']:
    // a stride-1 convolution of dY (K channels, P x Q image) producing the H x W grid.
    ConvGeom g = make_geom(dy, N, K, P, Q, R, S, 1, R - 1 - pad, H, W);
    if (S - 1 - pad != R - 1 - pad) return hipErrorInvalidValue;  // square windows only
    GatherKParams wa;
    wa.base = w; wa.rows = C; wa.rstride = R * S; wa.kstride = C * R * S; wa.rs = R * S; wa.flip = 1;
    wa.fd_rs = make_fastdiv((uint32_t)(R * S));
    ConvOut eo;
    eo.out = dx; eo.mask = relu_mask; eo.rows = C; eo.M = g.M; eo.PQ = H * W; eo.relu = 0; eo.fd_pq = g.fd_pq;
    if (is_winograd(use)) return conv_winograd(dy, w, (float*)ws, dx, relu_mask, 0, N, K, H, W, C, K, C, 1, winograd_tile(use), winograd_small(use), st);
    if (use == kKernelPacked) return conv_fast(dy, w, (float*)ws, eo, N, K, P, Q, K, C, R, S, 1, R - 1 - pad, H, W, 1, st);
    return conv_gemm(wa, g, eo, st);
}

// -------------------------------------------------------------------------------------------
// convolution backward-filter
// -------------------------------------------------------------------------------------------
// Fast path: input channels a multiple of 32 (a column tile of 32, 64, 96 or 128 columns that divides C never
// straddles two filter taps), both tensors below 4 GiB.  It always goes through the workspace (the column order there is
// tap-major and the final pass permutes it back), so the workspace is max(splits, 1) copies of dW.
static bool bwdf_fast_ok(int N, int C, int H, int W, int K, int P, int Q) {
    return C % 32 == 0 && (long long)N * C * H * W * 4 < 0xfffffff0LL && (long long)N * K * P * Q * 4 < 0xfffffff0LL;
}

// 64-channel layers run column tiles of three taps (192 columns); their split count follows from that tile count.
static bool bwdf_three_taps(int C, int R, int S) { return C == 64 && (R * S) % 3 == 0; }

static int bwdf_splits(int N, int C, int H, int W, int K, int R, int S, int P, int Q) {
    const long long M = (long long)N * P * Q;
    if (bwdf_fast_ok(N, C, H, W, K, P, Q) && bwdf_three_taps(C, R, S)) {
        const long long tiles = (long long)cdiv(K, K <= 64 ? 64 : 128) * (R * S / 3);
        return (int)std::max<long long>(1, std::min<long long>(1024 / tiles, cdiv(M, kMinReduction)));
    }
    return gemm_splits(K, (long long)C * R * S, M);
}

// workspace of the direct backward-filter kernels
size_t conv_bwd_filter_packed_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (bwdf_fast_ok(N, C, H, W, K, P, Q))
        return (size_t)bwdf_splits(N, C, H, W, K, R, S, P, Q) * K * C * R * S * sizeof(float);
    return gemm_workspace_bytes(K, (long long)C * R * S, (long long)N * P * Q);
}

// Winograd backward-filter (winograd.h): same geometry as the other two passes, input channels a multiple of 128 (the
// column tile of the grouped GEMM), 256 or more output channels (128 -> 256 measured 158 against 131 TFLOP/s).
// Workspace: the 16 accumulated products dU [16][K][C], their per-split partial sums [16][splits][K][C], then V and Dt
// for a chunk of images.
static bool wino_bwdf_ok(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int m) {
    return R == 3 && S == 3 && stride == 1 && pad == 1 && C % 128 == 0 && K >= (m == 4 ? 128 : 256) && N >= 1 && C <= 65535 && K <= 65535 &&
           (long long)wino_tiles(H, W, m) <= 32768 && (long long)H * W <= (1 << 24);
}

static int wino_bwdf_splits(int nb, int T, int K, int C, int m) {
    return (int)std::max<long long>(1, std::min<long long>(wino_bwdf_max_splits(K, C, m), cdiv((long long)nb * T, 512)));
}

static size_t wino_bwdf_workspace(int N, int C, int H, int W, int K, int m, bool small) {
    const int T = wino_tiles(H, W, m), nb = wino_chunk(N, C, H, W, K, m, small, true), G = wino_groups(m);
    return (size_t)G * K * C * sizeof(float) * (1 + wino_bwdf_splits(nb, T, K, C, m)) + (size_t)nb * G * (C + K) * T * sizeof(float);
}

size_t conv_bwd_filter_workspace(int N, int C, int H, int W, int K, int R, int S, int stride, int pad) {
    return fastest_workspace(kPassBwdFilter, N, C, H, W, K, R, S, stride, pad);
}

template <int BM, int BN, int WM, int WN, int BK = 32, int TAPS = 1>
static hipError_t bwdf_fast_cfg(BwdFilterFastParams& p, hipStream_t st) {
    auto kern = conv_bwdf_fast_kernel<BM, BN, WM, WN, BK, TAPS>;
    constexpr int PAD = BK >= 32 ? 1 : 32 / BK;  // as in the kernel
    constexpr size_t smem = sizeof(float) * 2 * BK * ((BM + PAD) + (BN + PAD));
    static std::atomic<bool> attr_set{false};
    if (hipError_t e = allow_smem(attr_set, (const void*)kern, smem); e != hipSuccess) return e;
    p.tiles_m = cdiv(p.K, BM);
    p.tiles_n = p.C * p.R * p.S / BN;
    p.ksplit = cdiv(cdiv(p.M, p.splits), BK) * BK;
    const long long nb = (long long)p.tiles_m * p.tiles_n * p.splits * p.groups;
    if (nb <= 0 || nb > 0x7fffffffLL) return hipErrorInvalidValue;
    VDNN_LAUNCH(kern, dim3((unsigned)nb), dim3(kThreads), smem, st, p);
    return hipGetLastError();
}

template <int BM, int BN, int WM, int WN>
static hipError_t bwdf_cfg(const PixKParams& pa, const ConvGeom& g, const RowMajorOut& eo, int splits, hipStream_t st) {
    constexpr int BK = 32, PAD = 1;
    return launch_tile<BM, BN, BK, WM, WN, PAD, PAD, PixK<BM, BK, PAD>, Im2colK<BN, BK, PAD>, RowMajorOut>(
        pa, g, eo, eo.rows, eo.cols, g.M, splits, st);
}

// x [N][C][H][W], dy [N][K][H][W] -> dw [K][C][3][3] through the grouped products of the Winograd form
static hipError_t conv_bwdf_winograd(const float* x, const float* dy, float* dw, float* ws, int N, int C, int H, int W, int K, int m, bool small,
                                     hipStream_t st) {
    const int T = wino_tiles(H, W, m), G = wino_groups(m);
    const int nb = wino_chunk(N, C, H, W, K, m, small, true);
    const int splits = wino_bwdf_splits(nb, T, K, C, m);
    const size_t kc = (size_t)K * C;
    float* acc = ws;
    float* part = acc + G * kc;
    float* v = part + (size_t)G * splits * kc;
    float* dt = v + (size_t)G * nb * C * T;
    const int rblocks = (int)std::min<size_t>((G * kc + 255) / 256, 8192);
    for (int n0 = 0; n0 < N; n0 += nb) {
        const int cur = std::min(nb, N - n0);
        hipError_t e = wino_input(x, v, n0, cur, C, H, W, m, st);
        if (e != hipSuccess) return e;
        if (m == 4) VDNN_LAUNCH(wino4_dy_kernel, dim3((unsigned)cdiv(K * T, 256), (unsigned)cur), dim3(256), 0, st, dy, dt, n0, cur, K, H, W);
        else VDNN_LAUNCH(wino_dy_kernel, dim3((unsigned)cdiv(K * T, 256), (unsigned)cur), dim3(256), 0, st, dy, dt, n0, cur, K, H, W);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        BwdFilterFastParams fp;
        fp.x = v; fp.dy = dt; fp.ws = part;
        fp.x_bytes = (uint32_t)((size_t)cur * C * T * 4);
        fp.dy_bytes = (uint32_t)((size_t)cur * K * T * 4);
        fp.K = K; fp.C = C; fp.H = cdiv(H, m); fp.W = cdiv(W, m); fp.R = 1; fp.S = 1; fp.stride = 1; fp.pad = 0; fp.P = cdiv(H, m); fp.Q = cdiv(W, m);
        fp.M = cur * T;
        fp.fd_pq = make_fastdiv((uint32_t)T);
        fp.fd_q = make_fastdiv((uint32_t)cdiv(W, m));
        fp.splits = splits;
        fp.groups = G;
        fp.x_gstride = (size_t)cur * C * T;
        fp.dy_gstride = (size_t)cur * K * T;
        fp.ws_gstride = (size_t)splits * kc;
        e = bwdf_fast_cfg<128, 128, 2, 2, 16>(fp, st);
        if (e != hipSuccess) return e;
        VDNN_LAUNCH(wino_accum_kernel, dim3((unsigned)rblocks), dim3(256), 0, st, (const float*)part, acc, kc, splits, G, n0 == 0 ? 1 : 0);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (m == 4) VDNN_LAUNCH(wino4_filter_grad_kernel, dim3((unsigned)std::min<size_t>((kc + 255) / 256, 8192)), dim3(256), 0, st, (const float*)acc, dw, kc);
    else VDNN_LAUNCH(wino_filter_grad_kernel, dim3((unsigned)std::min<size_t>((kc + 255) / 256, 8192)), dim3(256), 0, st, (const float*)acc, dw, kc);
    return hipGetLastError();
}

hipError_t conv_bwd_filter(const float* x, const float* dy, float* dw, void* ws, size_t ws_bytes, int N, int C, int H, int W,
                           int K, int R, int S, int stride, int pad, int kernel, hipStream_t st) {
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (P <= 0 || Q <= 0) return hipErrorInvalidValue;
    if (!fits_i32((long long)N * C * H * W) || !fits_i32((long long)N * K * P * Q)) return hipErrorInvalidValue;
    const int use = resolve_kernel(kPassBwdFilter, kernel, ws, ws_bytes, N, C, H, W, K, R, S, stride, pad);
    if (use == -2) return hipErrorInvalidValue;
    if (is_winograd(use)) return conv_bwdf_winograd(x, dy, dw, (float*)ws, N, C, H, W, K, winograd_tile(use), winograd_small(use), st);
    const int CRS = C * R * S;
    int splits = bwdf_splits(N, C, H, W, K, R, S, P, Q);
    const bool have_ws = use == kKernelPacked;
    if (!have_ws) splits = 1;  // memory-optimal algorithm: no workspace, the whole reduction in one workgroup per tile
    if (have_ws && bwdf_fast_ok(N, C, H, W, K, P, Q)) {
        BwdFilterFastParams fp;
        fp.x = x; fp.dy = dy; fp.ws = (float*)ws;
        fp.x_bytes = (uint32_t)((size_t)N * C * H * W * 4);
        fp.dy_bytes = (uint32_t)((size_t)N * K * P * Q * 4);
        fp.K = K; fp.C = C; fp.H = H; fp.W = W; fp.R = R; fp.S = S; fp.stride = stride; fp.pad = pad; fp.P = P; fp.Q = Q;
        fp.M = N * P * Q;
        fp.fd_pq = make_fastdiv((uint32_t)(P * Q));
        fp.fd_q = make_fastdiv((uint32_t)Q);
        fp.splits = splits;
        hipError_t e;
        // K-step 16 (33 KB of LDS, 4 workgroups per CU) for the 128-row tiles, 32 for the 64-row ones: measured
        // 127 against 121 TFLOP/s on VGG-16's 128..512-channel layers, 105 against 94 on the 64-channel one
        // column tiles lie inside one tap, so their width divides C: 128, else 96 or 64, else 32
        if (C % 128 == 0) e = K <= 64 ? bwdf_fast_cfg<64, 128, 1, 4, 32>(fp, st) : bwdf_fast_cfg<128, 128, 2, 2, 16>(fp, st);
        else if (bwdf_three_taps(C, R, S))  // 64-channel layers: tiles of three taps (192 columns) instead of one
            e = K <= 64 ? bwdf_fast_cfg<64, 192, 2, 2, 16, 3>(fp, st) : bwdf_fast_cfg<128, 192, 2, 2, 16, 3>(fp, st);
        else if (C % 96 == 0) e = bwdf_fast_cfg<128, 96, 4, 1, 16>(fp, st);
        else if (C % 64 == 0) e = K <= 64 ? bwdf_fast_cfg<64, 64, 2, 2, 32>(fp, st) : bwdf_fast_cfg<128, 64, 4, 1, 16>(fp, st);
        else e = bwdf_fast_cfg<128, 32, 4, 1, 16>(fp, st);
        if (e != hipSuccess) return e;
        return launch_reduce((const float*)ws, dw, (size_t)K * CRS, splits, st, C, R * S);  // adds the splits, [k][tap][c] -> [k][c][tap]
    }
    ConvGeom g = make_geom(x, N, C, H, W, R, S, stride, pad, P, Q);
    PixKParams pa;
    pa.base = dy; pa.rows = K; pa.PQ = P * Q; pa.fd_pq = g.fd_pq;
    RowMajorOut eo;
    eo.out = splits > 1 ? (float*)ws : dw;
    eo.rows = K; eo.cols = CRS; eo.ld = CRS; eo.slice = (size_t)K * CRS;
    // a first layer has few columns (C*R*S = 27 for RGB 3x3): narrow column tiles waste less of the matrix pipe
    hipError_t e;
    if (CRS <= 64) e = K <= 64 ? bwdf_cfg<64, 64, 2, 2>(pa, g, eo, splits, st) : bwdf_cfg<128, 64, 4, 1>(pa, g, eo, splits, st);
    else e = K <= 64 ? bwdf_cfg<64, 128, 1, 4>(pa, g, eo, splits, st) : bwdf_cfg<128, 128, 2, 2>(pa, g, eo, splits, st);
    if (e != hipSuccess) return e;
    if (splits > 1) return launch_reduce((const float*)ws, dw, (size_t)K * CRS, splits, st);
    return hipSuccess;
}

// -------------------------------------------------------------------------------------------
// backward-filter on a workspace that nobody allocates
// -------------------------------------------------------------------------------------------
// For callers that cannot allocate (under HIP graph capture, in a serving loop, in a harness that forbids it): the
// workspace of the backward-filter kernels (partial sums of the split reduction, Winograd transforms) lives in a
// file-scope device array.  Every GPU the library runs on holds its own copy of the array until the process ends.
// In host code the array's name is only a stand-in for the symbol: its device address is looked up once per device,
// with that device current, and kept; launches and anything else that needs the memory use that address.
// The kernels write every workspace word they later read (the existing entry point runs on uninitialised workspaces
// too), so nothing has to be cleared between calls; two calls that overlap on one GPU share the array and race.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static hipError_t static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // two threads racing here look up the same address
    }
    *out = p;
    return hipSuccess;
}

// kernel: kKernelAuto = the fastest kernel that applies to the shape (what conv_bwd_filter_workspace sizes for).
// *need receives the workspace bytes of the kernel in question; hipErrorInvalidValue with *need > kStaticScratchBytes
// means "too large for the static buffer" (nothing is launched).
hipError_t conv_bwd_filter_static(const float* x, const float* dy, float* dw, int N, int C, int H, int W, int K, int R, int S, int stride,
                                  int pad, int kernel, hipStream_t st, size_t* need) {
    int use = kernel;
    if (kernel == kKernelAuto) {
        use = kKernelGather;
        for (int k : kAutoOrder)
            if (conv_workspace(kPassBwdFilter, k, N, C, H, W, K, R, S, stride, pad) != kNoKernel) { use = k; break; }
    }
    *need = conv_workspace(kPassBwdFilter, use, N, C, H, W, K, R, S, stride, pad);
    if (*need == kNoKernel) { *need = 0; return hipErrorInvalidValue; }
    if (*need > kStaticScratchBytes) return hipErrorInvalidValue;
    void* ws = nullptr;
    hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return e;
    return conv_bwd_filter(x, dy, dw, ws, kStaticScratchBytes, N, C, H, W, K, R, S, stride, pad, use, st);
}

// -------------------------------------------------------------------------------------------
// FC
// -------------------------------------------------------------------------------------------
size_t fc_workspace(int N, int I, int O, int which) {
    if (which == 0) return gemm_workspace_bytes(N, O, I);
    if (which == 1) return gemm_workspace_bytes(N, I, O);
    return gemm_workspace_bytes(O, I, N);
}

static GatherKParams dense_k(const float* base, int rows, int ld) {
    GatherKParams p;
    p.base = base; p.rows = rows; p.rstride = ld; p.kstride = 1; p.rs = 1; p.flip = 0;
    p.fd_rs = make_fastdiv(1);
    return p;
}

static RowMajorOut fc_out(float* out, void* ws, int rows, int cols, int splits) {
    RowMajorOut eo;
    eo.out = splits > 1 ? (float*)ws : out;
    eo.rows = rows; eo.cols = cols; eo.ld = cols; eo.slice = (size_t)rows * cols;
    return eo;
}

hipError_t fc_fwd(const float* x, const float* w, float* y, void* ws, size_t ws_bytes, int N, int I, int O, hipStream_t st) {
    constexpr int BK = 16, PAD = 2;
    const int splits = (ws && ws_bytes >= gemm_workspace_bytes(N, O, I)) ? gemm_splits(N, O, I) : 1;
    RowMajorOut eo = fc_out(y, ws, N, O, splits);
    hipError_t e = launch_tile<128, 128, BK, 2, 2, PAD, PAD, GatherK<128, BK, PAD>, GatherK<128, BK, PAD>, RowMajorOut>(
        dense_k(x, N, I), dense_k(w, O, I), eo, N, O, I, splits, st);
    if (e != hipSuccess) return e;
    return splits > 1 ? launch_reduce((const float*)ws, y, (size_t)N * O, splits, st) : hipSuccess;
}

hipError_t fc_bwd_data(const float* dy, const float* w, float* dx, void* ws, size_t ws_bytes, int N, int I, int O, hipStream_t st) {
    constexpr int BK = 16, PADA = 2, PADB = 32;
    const int splits = (ws && ws_bytes >= gemm_workspace_bytes(N, I, O)) ? gemm_splits(N, I, O) : 1;
    RowMajorOut eo = fc_out(dx, ws, N, I, splits);
    DenseRParams pb;
    pb.base = w; pb.rows = I; pb.ld = I;
    hipError_t e = launch_tile<128, 128, BK, 2, 2, PADA, PADB, GatherK<128, BK, PADA>, DenseR<128, BK, PADB>, RowMajorOut>(
        dense_k(dy, N, O), pb, eo, N, I, O, splits, st);
    if (e != hipSuccess) return e;
    return splits > 1 ? launch_reduce((const float*)ws, dx, (size_t)N * I, splits, st) : hipSuccess;
}

hipError_t fc_bwd_filter(const float* x, const float* dy, float* dw, void* ws, size_t ws_bytes, int N, int I, int O, hipStream_t st) {
    constexpr int BK = 16, PAD = 32;
    const int splits = (ws && ws_bytes >= gemm_workspace_bytes(O, I, N)) ? gemm_splits(O, I, N) : 1;
    RowMajorOut eo = fc_out(dw, ws, O, I, splits);
    DenseRParams pa, pb;
    pa.base = dy; pa.rows = O; pa.ld = O;
    pb.base = x; pb.rows = I; pb.ld = I;
    hipError_t e = launch_tile<128, 128, BK, 2, 2, PAD, PAD, DenseR<128, BK, PAD>, DenseR<128, BK, PAD>, RowMajorOut>(
        pa, pb, eo, O, I, N, splits, st);
    if (e != hipSuccess) return e;
    return splits > 1 ? launch_reduce((const float*)ws, dw, (size_t)O * I, splits, st) : hipSuccess;
}

}  // namespace vdnn
