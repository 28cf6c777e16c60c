// LDS-tiled fp32 MFMA GEMM core for gfx950 (64-wide wavefronts, v_mfma_f32_32x32x2_f32).
//
// One workgroup of 256 threads (4 waves) computes a BM x BN tile of D = A * B^T-like products,
// where the two operands are fetched by "loader" policies.  The loaders are what turn this one
// core into convolution forward / backward-data (implicit GEMM: the B operand is gathered from
// the feature map, never materialised), convolution backward-filter (both operands indexed by
// pixel along the reduction) and the three FC products.
//
// Data flow per K-step of BK: global -> registers (issued one step ahead) -> LDS (double
// buffered, k-major so that the 32 lanes of an MFMA operand read 32 consecutive words: no bank
// conflicts) -> MFMA.  One barrier per K-step.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vdnn {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;

// Division by a runtime constant: q = (mulhi(n, m) + n) >> s, exact for n < 2^31.
struct FastDiv {
    uint32_t d, m, s;
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    f.s = s;
    f.m = (uint32_t)((((1ull << 32) * ((1ull << s) - d)) / d) + 1);
    return f;
}

__device__ __forceinline__ uint32_t fd_div(uint32_t n, const FastDiv& f) { return (__umulhi(n, f.m) + n) >> f.s; }

// ---------------------------------------------------------------------------------------------
// Thread -> element mappings for filling a ROWS x BK operand tile with 256 threads.
//   RowFast: consecutive lanes walk along rows   (used when global memory is row-contiguous)
//   KFast  : consecutive lanes walk along k      (used when global memory is k-contiguous)
// LDS layout of a tile is always tile[kk * (ROWS + PAD) + row].
// ---------------------------------------------------------------------------------------------
template <int ROWS, int BK>
struct RowFast {
    static_assert(ROWS == 32 || ROWS == 64 || ROWS == 128 || ROWS == 256, "tile rows");
    static constexpr int E = ROWS * BK / kThreads;
    static constexpr int KSTEP = kThreads / ROWS > 0 ? kThreads / ROWS : 1;  // k distance between a thread's elements
    __device__ static int row(int tid) { return tid % ROWS; }
    __device__ static int kk0(int tid) { return tid / ROWS; }
};

template <int ROWS, int BK>
struct KFast {
    static constexpr int E = ROWS * BK / kThreads;
    static constexpr int RSTEP = kThreads / BK;  // row distance between a thread's elements
    static_assert(kThreads % BK == 0 && (ROWS * BK) % kThreads == 0, "tile shape");
    __device__ static int kk(int tid) { return tid % BK; }
    __device__ static int row0(int tid) { return tid / BK; }
};

// ---------------------------------------------------------------------------------------------
// Loaders.  Each has Params (host-filled, passed by value), per-thread state set by init(), and
//   load(regs, k0, kend): fetch this thread's elements of the tile whose reduction index starts at k0;
//   store(tile, regs)   : write them to the LDS tile.
// Elements outside the matrix (row >= rows, k >= kend, padding of the image) read as 0.
// ---------------------------------------------------------------------------------------------

// Matrix stored with the reduction index fastest, optionally through a (k / rs, k % rs) split:
//   element(row, k) = base[row * rstride + (k / rs) * kstride + rs_index], rs_index = k % rs, or
//   rs - 1 - k % rs when flip is set.
// rs = 1, kstride = 1 is a plain row-major matrix (W[K][C*R*S] for forward, FC operands).  With
// rs = R*S, rstride = R*S, kstride = C*R*S and flip it reads W[k][c][R-1-r][S-1-s] as a matrix
// indexed [c][(k, r, s)]: the operand of backward-data, with no transposed copy of W in memory.
struct GatherKParams {
    const float* base;
    int rows;
    int rstride, kstride, rs, flip;
    FastDiv fd_rs;
};

template <int ROWS, int BK, int PAD>
struct GatherK {
    using Map = KFast<ROWS, BK>;
    using Params = GatherKParams;
    static constexpr int E = Map::E;
    const float* base;
    int row_first, kk;
    __device__ void init(const Params& p, int tile_row0, int tid) {
        base = p.base;
        kk = Map::kk(tid);
        row_first = tile_row0 + Map::row0(tid);
    }
    __device__ void load(const Params& p, float (&r)[E], int k0, int kend) {
        const int k = k0 + kk;
        const bool okk = k < kend;
        const uint32_t kq = fd_div((uint32_t)k, p.fd_rs);
        int rs = k - (int)kq * p.rs;
        if (p.flip) rs = p.rs - 1 - rs;
        const int koff = (int)kq * p.kstride + rs;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int row = row_first + j * Map::RSTEP;
            const bool ok = okk && row < p.rows;
            r[j] = ok ? base[(size_t)row * p.rstride + koff] : 0.f;
        }
    }
    __device__ void store(float* tile, const float (&r)[E], int tid) {
        const int kkl = Map::kk(tid), r0 = Map::row0(tid);
#pragma unroll
        for (int j = 0; j < E; ++j) tile[kkl * (ROWS + PAD) + r0 + j * Map::RSTEP] = r[j];
    }
};

// Matrix stored with the row index fastest: element(row, k) = base[k * ld + row].
struct DenseRParams {
    const float* base;
    int rows, ld;
};

template <int ROWS, int BK, int PAD>
struct DenseR {
    using Map = RowFast<ROWS, BK>;
    using Params = DenseRParams;
    static constexpr int E = Map::E;
    int row, kk0;
    bool vrow;
    __device__ void init(const Params& p, int tile_row0, int tid) {
        row = tile_row0 + Map::row(tid);
        vrow = row < p.rows;
        kk0 = Map::kk0(tid);
    }
    __device__ void load(const Params& p, float (&r)[E], int k0, int kend) {
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int k = k0 + kk0 + j * Map::KSTEP;
            r[j] = (vrow && k < kend) ? p.base[(size_t)k * p.ld + row] : 0.f;
        }
    }
    __device__ void store(float* tile, const float (&r)[E], int tid) {
        const int rl = Map::row(tid), k0 = Map::kk0(tid);
#pragma unroll
        for (int j = 0; j < E; ++j) tile[(k0 + j * Map::KSTEP) * (ROWS + PAD) + rl] = r[j];
    }
};

// Geometry of a convolution seen as a gather: rows are output pixels m = (n, p, q), the reduction
// index is k = (c, r, s); element(m, k) = src[n][c][p*stride - pad + r][q*stride - pad + s], zero
// outside the image.  Forward uses it on X; backward-data (stride 1) uses it on dY with
// pad' = R - 1 - pad and the filter taps flipped on the weight side.
struct ConvGeom {
    const float* src;
    int C, H, W;        // source tensor channels and image size
    int R, S, stride, pad;
    int P, Q;           // pixel grid of the rows
    int M;              // N * P * Q
    int Ktot;           // C * R * S
    FastDiv fd_pq, fd_q, fd_rs, fd_s;
};

// Rows = pixels, lanes walk along pixels (contiguous in NCHW for stride 1).
template <int ROWS, int BK, int PAD>
struct Im2colR {
    using Map = RowFast<ROWS, BK>;
    using Params = ConvGeom;
    static constexpr int E = Map::E;
    static_assert(ROWS >= 64, "k index must be uniform per wave");
    int pix_off, ih0, iw0, kk0;
    bool vm;
    __device__ void init(const Params& g, int tile_row0, int tid) {
        const int m = tile_row0 + Map::row(tid);
        vm = m < g.M;
        const uint32_t mm = vm ? (uint32_t)m : 0u;
        const uint32_t n = fd_div(mm, g.fd_pq);
        const uint32_t pq = mm - n * (uint32_t)(g.P * g.Q);
        const uint32_t p = fd_div(pq, g.fd_q);
        const uint32_t q = pq - p * (uint32_t)g.Q;
        ih0 = (int)p * g.stride - g.pad;
        iw0 = (int)q * g.stride - g.pad;
        pix_off = (int)n * g.C * g.H * g.W + ih0 * g.W + iw0;
        // tid / ROWS is the same for all lanes of a wave when ROWS >= 64: keep it in a scalar register
        kk0 = __builtin_amdgcn_readfirstlane(Map::kk0(tid));
    }
    __device__ void load(const Params& g, float (&r)[E], int k0, int kend) {
        const int RS = g.R * g.S, HW = g.H * g.W;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int k = k0 + kk0 + j * Map::KSTEP;  // wave-uniform
            const uint32_t c = fd_div((uint32_t)k, g.fd_rs);
            const uint32_t rs = (uint32_t)k - c * (uint32_t)RS;
            const uint32_t rr = fd_div(rs, g.fd_s);
            const uint32_t ss = rs - rr * (uint32_t)g.S;
            const int ih = ih0 + (int)rr, iw = iw0 + (int)ss;
            const bool ok = vm && k < kend && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
            r[j] = ok ? g.src[pix_off + (int)c * HW + (int)rr * g.W + (int)ss] : 0.f;
        }
    }
    __device__ void store(float* tile, const float (&r)[E], int tid) {
        const int rl = Map::row(tid), k0 = Map::kk0(tid);
#pragma unroll
        for (int j = 0; j < E; ++j) tile[(k0 + j * Map::KSTEP) * (ROWS + PAD) + rl] = r[j];
    }
};

// Backward-filter operand B: rows = (c, r, s), reduction index = pixel m; lanes walk along pixels.
// element(row, m) = X[n][c][p*stride - pad + r][q*stride - pad + s].
template <int ROWS, int BK, int PAD>
struct Im2colK {
    using Map = KFast<ROWS, BK>;
    using Params = ConvGeom;
    static constexpr int E = Map::E;
    int kk;
    int koff[E];   // c*H*W + r*W + s of this thread's rows
    int rs_pack[E];  // (r << 16) | s, or -1 when the row is outside the matrix
    __device__ void init(const Params& g, int tile_row0, int tid) {
        kk = Map::kk(tid);
        const int RS = g.R * g.S, HW = g.H * g.W;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int row = tile_row0 + Map::row0(tid) + j * Map::RSTEP;
            const bool ok = row < g.Ktot;
            const uint32_t rw = ok ? (uint32_t)row : 0u;
            const uint32_t c = fd_div(rw, g.fd_rs);
            const uint32_t rs = rw - c * (uint32_t)RS;
            const uint32_t rr = fd_div(rs, g.fd_s);
            const uint32_t ss = rs - rr * (uint32_t)g.S;
            koff[j] = (int)c * HW + (int)rr * g.W + (int)ss;
            rs_pack[j] = ok ? (int)((rr << 16) | ss) : -1;
        }
    }
    __device__ void load(const Params& g, float (&r)[E], int k0, int kend) {
        const int m = k0 + kk;
        const bool vm = m < kend;
        const uint32_t mm = vm ? (uint32_t)m : 0u;
        const uint32_t n = fd_div(mm, g.fd_pq);
        const uint32_t pq = mm - n * (uint32_t)(g.P * g.Q);
        const uint32_t p = fd_div(pq, g.fd_q);
        const uint32_t q = pq - p * (uint32_t)g.Q;
        const int ih0 = (int)p * g.stride - g.pad, iw0 = (int)q * g.stride - g.pad;
        const int pix_off = (int)n * g.C * g.H * g.W + ih0 * g.W + iw0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int ih = ih0 + (rs_pack[j] >> 16), iw = iw0 + (rs_pack[j] & 0xffff);
            const bool ok = vm && rs_pack[j] >= 0 && (unsigned)ih < (unsigned)g.H && (unsigned)iw < (unsigned)g.W;
            r[j] = ok ? g.src[pix_off + koff[j]] : 0.f;
        }
    }
    __device__ void store(float* tile, const float (&r)[E], int tid) {
        const int kkl = Map::kk(tid), r0 = Map::row0(tid);
#pragma unroll
        for (int j = 0; j < E; ++j) tile[kkl * (ROWS + PAD) + r0 + j * Map::RSTEP] = r[j];
    }
};

// Backward-filter operand A: rows = output channel k, reduction index = pixel m = (n, p, q);
// element(k, m) = dY[n][k][p][q]; lanes walk along pixels.
struct PixKParams {
    const float* base;
    int rows;  // K
    int PQ;
    FastDiv fd_pq;
};

template <int ROWS, int BK, int PAD>
struct PixK {
    using Map = KFast<ROWS, BK>;
    using Params = PixKParams;
    static constexpr int E = Map::E;
    int kk, row_first;
    __device__ void init(const Params& p, int tile_row0, int tid) {
        kk = Map::kk(tid);
        row_first = tile_row0 + Map::row0(tid);
    }
    __device__ void load(const Params& p, float (&r)[E], int k0, int kend) {
        const int m = k0 + kk;
        const bool vm = m < kend;
        const uint32_t mm = vm ? (uint32_t)m : 0u;
        const uint32_t n = fd_div(mm, p.fd_pq);
        const uint32_t pq = mm - n * (uint32_t)p.PQ;
        const size_t off = (size_t)n * p.rows * p.PQ + pq;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int row = row_first + j * Map::RSTEP;
            r[j] = (vm && row < p.rows) ? p.base[off + (size_t)row * p.PQ] : 0.f;
        }
    }
    __device__ void store(float* tile, const float (&r)[E], int tid) {
        const int kkl = Map::kk(tid), r0 = Map::row0(tid);
#pragma unroll
        for (int j = 0; j < E; ++j) tile[kkl * (ROWS + PAD) + r0 + j * Map::RSTEP] = r[j];
    }
};

// ---------------------------------------------------------------------------------------------
// Epilogues: where element (row, col) of the tile goes.
// ---------------------------------------------------------------------------------------------

// Row-major matrix D[row * ld + col]; reduction split s writes its partial sums at out + s * slice.
struct RowMajorOut {
    float* out;
    int rows, cols, ld;
    size_t slice;
    struct Col {
        size_t off;
        bool ok;
    };
    __device__ Col col(int c) const { return Col{(size_t)c, c < cols}; }
    __device__ void put(float* base, int row, const Col& c, float v) const {
        if (c.ok && row < rows) base[(size_t)row * ld + c.off] = v;
    }
    __device__ float* base(int split) const { return out + (size_t)split * slice; }
};

// NCHW feature map: row = channel k, col = pixel m = (n, pq) -> Y[(n*K + k)*PQ + pq]; optional ReLU
// on the value (forward), or optional zeroing where a same-shaped tensor is not positive (backward-data
// with the backward of the preceding in-place ReLU folded in: mask = that ReLU's output).
struct ConvOut {
    float* out;
    const float* mask;
    int rows;  // K
    int M, PQ;
    int relu;
    FastDiv fd_pq;
    struct Col {
        size_t off;
        bool ok;
    };
    __device__ Col col(int m) const {
        const bool ok = m < M;
        const uint32_t mm = ok ? (uint32_t)m : 0u;
        const uint32_t n = fd_div(mm, fd_pq);
        const uint32_t pq = mm - n * (uint32_t)PQ;
        return Col{(size_t)n * rows * PQ + pq, ok};
    }
    __device__ void put(float* base, int row, const Col& c, float v) const {
        if (relu) v = v > 0.f ? v : 0.f;
        if (c.ok && row < rows) {
            const size_t idx = c.off + (size_t)row * PQ;
            if (mask && !(mask[idx] > 0.f)) v = 0.f;
            base[idx] = v;
        }
    }
    // Two neighbouring pixels (c1 is the column after c0, c0's pixel index even) of one row: a single 8-byte store
    // when both lie in the same image plane at an even offset, two plain stores otherwise.
    __device__ void put2(float* base, int row, const Col& c0, const Col& c1, float v0, float v1) const {
        if (c1.ok && c1.off == c0.off + 1 && !(PQ & 1) && !(c0.off & 1)) {
            if (relu) v0 = v0 > 0.f ? v0 : 0.f, v1 = v1 > 0.f ? v1 : 0.f;
            if (row < rows) {
                const size_t idx = c0.off + (size_t)row * PQ;
                if (mask) {
                    const float2 m = *reinterpret_cast<const float2*>(mask + idx);
                    if (!(m.x > 0.f)) v0 = 0.f;
                    if (!(m.y > 0.f)) v1 = 0.f;
                }
                *reinterpret_cast<float2*>(base + idx) = make_float2(v0, v1);
            }
        } else {
            put(base, row, c0, v0);
            put(base, row, c1, v1);
        }
    }
    __device__ float* base(int) const { return out; }
};

// ---------------------------------------------------------------------------------------------
// The kernel.  Grid is 1-D: tiles_m * tiles_n * splits workgroups.  Consecutive workgroup ids are
// dealt round-robin to the 8 XCDs (each with its own L2), so ids are first permuted such that each
// XCD gets a contiguous run of logical tiles; within a run, tiles that differ only in the row tile
// (same pixels / same reduction slice) are adjacent and share their big operand through that L2.
// ---------------------------------------------------------------------------------------------
struct GridInfo {
    int tiles_m, tiles_n, splits;
    int ktot, ksplit;  // reduction length and per-split length (multiple of BK)
};

__device__ __forceinline__ int xcd_remap(int bid, int nb) {
    const int per = nb >> 3, rem = nb & 7;
    const int xcd = bid & 7, idx = bid >> 3;
    const int start = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
    return start + idx;
}

template <int BM, int BN, int BK, int WM, int WN, int PADA, int PADB, class LA, class LB, class EP>
__global__ __launch_bounds__(kThreads) void gemm_tile_kernel(typename LA::Params pa, typename LB::Params pb, EP ep,
                                                              GridInfo gi) {
    static_assert(WM * WN == 4, "4 waves");
    constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    static_assert(TM >= 1 && TN >= 1 && TM * WM * 32 == BM && TN * WN * 32 == BN, "wave tiling");
    static_assert(BK % 2 == 0, "k step of the MFMA");
    constexpr int LDA = BM + PADA, LDB = BN + PADB;
    extern __shared__ float smem[];
    float* As = smem;                 // [2][BK][LDA]
    float* Bs = smem + 2 * BK * LDA;  // [2][BK][LDB]

    const int tid = threadIdx.x;
    const int nb = gi.tiles_m * gi.tiles_n * gi.splits;
    const int logical = xcd_remap(blockIdx.x, nb);
    const int tiles = gi.tiles_m * gi.tiles_n;
    const int split = logical / tiles;
    const int t2 = logical - split * tiles;
    const int tile_n = t2 / gi.tiles_m, tile_m = t2 - tile_n * gi.tiles_m;
    const int row0 = tile_m * BM, col0 = tile_n * BN;
    const int kbeg = split * gi.ksplit;
    const int kend = min(gi.ktot, kbeg + gi.ksplit);

    LA la;
    LB lb;
    la.init(pa, row0, tid);
    lb.init(pb, col0, tid);

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int l32 = lane & 31, khalf = lane >> 5;
    const int a_off = khalf * LDA + wm * (TM * 32) + l32;
    const int b_off = khalf * LDB + wn * (TN * 32) + l32;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    float ra[LA::E], rb[LB::E];
    const int nk = (kend - kbeg + BK - 1) / BK;
    if (nk > 0) {
        la.load(pa, ra, kbeg, kend);
        lb.load(pb, rb, kbeg, kend);
        la.store(As, ra, tid);
        lb.store(Bs, rb, tid);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) {
            la.load(pa, ra, kbeg + (kt + 1) * BK, kend);
            lb.load(pb, rb, kbeg + (kt + 1) * BK, kend);
        }
        const float* at = As + cur * BK * LDA + a_off;
        const float* bt = Bs + cur * BK * LDB + b_off;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = at[kk * LDA + i * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = bt[kk * LDB + j * 32];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            la.store(As + (cur ^ 1) * BK * LDA, ra, tid);
            lb.store(Bs + (cur ^ 1) * BK * LDB, rb, tid);
        }
        __syncthreads();
    }

    // Accumulator layout of the 32x32 MFMA: register v of lane l holds D[8*(v/4) + 4*(l/32) + v%4][l%32].
    float* obase = ep.base(split);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const typename EP::Col c = ep.col(col0 + wn * (TN * 32) + j * 32 + l32);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int rbase = row0 + wm * (TM * 32) + i * 32 + 4 * khalf;
#pragma unroll
            for (int v = 0; v < 16; ++v) ep.put(obase, rbase + 8 * (v / 4) + (v % 4), c, acc[i][j][v]);
        }
    }
}

template <int BM, int BN, int BK, int PADA, int PADB>
constexpr size_t gemm_smem_bytes() {
    return sizeof(float) * 2 * BK * ((BM + PADA) + (BN + PADB));
}

}  // namespace vdnn
