// Fast path of the implicit-GEMM convolution (forward and stride-1 backward-data) for channel
// counts that are a multiple of 16.
//
// The reduction index is ordered (channel block of 16, filter tap, channel in block), so that one
// K-step of 16 lies inside a single filter tap: the tap decomposition and the image-border test
// happen once per K-step per thread instead of once per element, and the 9 taps of a 3x3 filter
// re-read the same 16 channels back to back (L1 hits).  Loads are raw buffer loads: the per-thread
// part of the address sits in a VGPR that never changes within a K-step, the per-element part in
// an SGPR, and elements outside the image (padding) or outside the matrix are redirected to an
// out-of-range offset for which the hardware returns 0 - no branches, no per-element vector ALU work.
// The weight operand is read from a packed copy Wp[k_ordered][row] (row = output channel for
// forward, input channel for backward-data) written by pack_weights_kernel just before, so
// that its tile loads are contiguous along rows.
#pragma once
#include "gemm_tile.h"

namespace vdnn {

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ float buf_load(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}

// 16 bytes; the address needs dword alignment only
__device__ __forceinline__ float4 buf_load4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0));
}

constexpr uint32_t kOobOffset = 0xfffffff0u;  // >= num_records of any buffer: the load returns 0

struct ConvFastParams {
    const float* src;   // X (forward) or dY (backward-data): [N][Cred][H][W]
    const float* wp;    // packed weights [Cred*R*S][rows]
    uint32_t src_bytes, wp_bytes;
    int rows;           // output channels of this GEMM
    int Cred, H, W;     // reduction channels and source image
    int R, S, stride, pad;
    int P, Q, M;        // output pixel grid, M = N*P*Q
    FastDiv fd_pq, fd_q;
    int tiles_m, tiles_n;
    // One launch covers the logical tiles [tile_begin, tile_begin + n_tiles).  With splits > 1 each tile's
    // reduction is cut into `splits` runs of `steps_per_split` K-steps, one workgroup each, and the raw
    // accumulators go to partial[(tile - tile_begin) * splits + split][BM][BN] instead of the output.
    int tile_begin, n_tiles, splits, steps_per_split;
    float* partial;
    ConvOut out;
    // groups > 1 (unsplit launches only): `groups` independent problems of the same shape in one launch, group g
    // reading src + g * src_gstride, wp + g * wp_gstride and writing out + g * out_gstride (strides in elements);
    // the grid is n_tiles * groups workgroups.  Used for the 16 element-wise products of the Winograd algorithm.
    int groups = 1;
    size_t src_gstride = 0, wp_gstride = 0, out_gstride = 0;
};

// Wp[((cb*RS + rs)*16 + ci)][row]:
//   forward:       row = k, value W[k][cb*16+ci][rs]                       (W is [K][C][R][S])
//   backward-data: row = c, value W[cb*16+ci][c][RS-1-rs]  (taps flipped, reduction over output channels)
__global__ void pack_weights_kernel(const float* __restrict__ w, float* __restrict__ wp, int K, int C, int RS, int bwd) {
    const int rows = bwd ? C : K;
    const size_t total = (size_t)K * C * RS;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int row = (int)(i % rows);
        const int kred = (int)(i / rows);
        const int ci = kred & 15, t = kred >> 4;
        const int rs = t % RS, cb = t / RS;
        const int ch = cb * 16 + ci;
        wp[i] = bwd ? w[((size_t)ch * C + row) * RS + (RS - 1 - rs)] : w[((size_t)row * C + ch) * RS + rs];
    }
}

// SPLIT = false: one workgroup per tile, whole reduction, result through the epilogue.
// SPLIT = true : one workgroup per (tile, split), partial sums to p.partial.
// 4 waves per SIMD (4 workgroups per CU: 128 registers per lane, 40 KB of LDS each for the 128x128 tile)
// keep the matrix pipe busier than the 3 the register allocator would settle for: 136-138 against 132-134 TFLOP/s
// (the same attribute on the backward-filter kernel measured no gain).
// Row pitch padding of the LDS tiles.  Lanes store consecutive rows and read 32 consecutive words, so no pitch
// conflicts; the 256-pixel tiles go without padding, which makes four of them (40 KB each) fit one CU's LDS.
template <int BN>
constexpr int kConvFastPad = BN >= 256 ? 0 : 32;

// QUAD = true (host-checked: rows a multiple of 4, 64+ rows per tile): a thread fetches four neighbouring weight rows
// with one 16-byte load and puts them to LDS with one 16-byte store (measured +0.5..1 %).  The same for four pixels of
// the gathered operand measured 4-5 % slower: two taps of three shift the pixels off 16-byte alignment.
template <int BM, int BN, int WM, int WN, bool SPLIT, bool QUAD = false>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void conv_fast_kernel(ConvFastParams p) {
    constexpr int BK = 16;
    constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "wave tiling");
    constexpr int PADA = kConvFastPad<BN>, PADB = kConvFastPad<BN>;
    constexpr int LDA = BM + PADA, LDB = BN + PADB;
    constexpr int EA = BM * BK / kThreads, EB = BN * BK / kThreads;
    constexpr int KSA = kThreads / BM > 0 ? kThreads / BM : 1;  // k distance between a thread's A elements
    constexpr int KSB = kThreads / BN > 0 ? kThreads / BN : 1;
    static_assert(EA >= 1 && EB >= 1, "tile too small");
    extern __shared__ __align__(16) float smem[];
    float* As = smem;
    float* Bs = smem + 2 * BK * LDA;

    const int tid = threadIdx.x;
    const int nsplit = SPLIT ? p.splits : 1;
    int logical = xcd_remap(blockIdx.x, p.n_tiles * nsplit * (SPLIT ? 1 : p.groups));
    // the same for the whole workgroup; said explicitly so that the buffer resources below stay in scalar registers
    const int group = SPLIT ? 0 : __builtin_amdgcn_readfirstlane(logical / p.n_tiles);
    if constexpr (!SPLIT) logical -= group * p.n_tiles;
    const int tile_local = logical / nsplit, split = logical - tile_local * nsplit;
    const int tile = (SPLIT ? p.tile_begin : 0) + tile_local;
    const int tile_n = tile / p.tiles_m, tile_m = tile - tile_n * p.tiles_m;
    const int row0 = tile_m * BM, col0 = tile_n * BN;

    const __amdgpu_buffer_rsrc_t rs_src = make_rsrc(p.src + (size_t)group * p.src_gstride, p.src_bytes);
    const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(p.wp + (size_t)group * p.wp_gstride, p.wp_bytes);

    // ---- A (weights): thread owns row a_row and k = a_k0 + j*KSA ----
    const int a_row = tid % BM, a_k0 = tid / BM;
    const uint32_t a_voff = (row0 + a_row < p.rows) ? (uint32_t)((a_k0 * p.rows + row0 + a_row) * 4) : kOobOffset;
    // ---- B (gathered feature map): thread owns pixel b_row and k = b_k0 + j*KSB ----
    const int b_row = tid % BN, b_k0 = tid / BN;
    const int HW = p.H * p.W;
    int ih0, iw0, pix_base;
    bool vm;
    {
        const int m = col0 + b_row;
        vm = m < p.M;
        const uint32_t mm = vm ? (uint32_t)m : 0u;
        const uint32_t n = fd_div(mm, p.fd_pq);
        const uint32_t pq = mm - n * (uint32_t)(p.P * p.Q);
        const uint32_t pp = fd_div(pq, p.fd_q);
        const uint32_t qq = pq - pp * (uint32_t)p.Q;
        ih0 = (int)pp * p.stride - p.pad;
        iw0 = (int)qq * p.stride - p.pad;
        pix_base = (int)n * p.Cred * HW + b_k0 * HW;  // + (ih*W + iw) of the tap
    }

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int l32 = lane & 31, khalf = lane >> 5;
    // A wave that owns two 32-wide MFMA blocks along a tile dimension interleaves them: block i takes the tile
    // positions 2*l + i of the wave's 64.  The two values a lane feeds to the two blocks then sit next to each
    // other in LDS, one 8-byte read with an immediate offset fetches both (no address arithmetic in the K loop),
    // and in the epilogue a lane holds two neighbouring pixels of each row.
    constexpr bool PAIR_M = TM == 2, PAIR_N = TN == 2;
    const int a_off = khalf * LDA + wm * (TM * 32) + (PAIR_M ? 2 * l32 : l32);
    const int b_off = khalf * LDB + wn * (TN * 32) + (PAIR_N ? 2 * l32 : l32);
    // tile row of element v of MFMA block i, tile column of this lane in MFMA block j
    auto tile_row = [&](int i, int v) {
        const int rr = 4 * khalf + 8 * (v / 4) + (v % 4);
        return wm * (TM * 32) + (PAIR_M ? 2 * rr + i : i * 32 + rr);
    };
    auto tile_col = [&](int j) { return wn * (TN * 32) + (PAIR_N ? 2 * l32 + j : j * 32 + l32); };
    float* a_st = As + a_k0 * LDA + a_row;
    float* b_st = Bs + b_k0 * LDB + b_row;

    // ---- QUAD: thread owns weight rows 4*aq .. 4*aq+3 and k = ak0 + j * KPA ----
    constexpr int QA = BM / 4;                 // quads per k row
    constexpr int KPA = kThreads / QA;         // k rows covered by one pass of the workgroup
    constexpr int NA = BK / KPA > 0 ? BK / KPA : 1;  // passes
    static_assert(!QUAD || (KPA <= BK && LDA % 4 == 0), "quad loads need 64+ rows per tile");
    const int aq = tid % QA, ak0 = tid / QA;
    const uint32_t a_voff4 = (row0 + 4 * aq < p.rows) ? (uint32_t)((ak0 * p.rows + row0 + 4 * aq) * 4) : kOobOffset;
    float4* a_st4 = reinterpret_cast<float4*>(As + ak0 * LDA + 4 * aq);

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int RS = p.R * p.S;
    const int total_steps = (p.Cred / 16) * RS;
    const int step_begin = SPLIT ? split * p.steps_per_split : 0;
    const int nsteps = SPLIT ? max(0, min(total_steps, step_begin + p.steps_per_split) - step_begin) : total_steps;
    // scalar state of the K-step being LOADED: channel block cb, tap (r, s)
    int cb = step_begin / RS;
    int r = (step_begin - cb * RS) / p.S;
    int s = step_begin - cb * RS - r * p.S;
    float ra[EA], rb[EB];

    auto load_step = [&](int step) {
        // tap and channel block are the same for the whole workgroup: what derives from them stays in scalar registers
        const int rr = __builtin_amdgcn_readfirstlane(r), ss = __builtin_amdgcn_readfirstlane(s);
        const uint32_t a_s = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)step * (uint32_t)(16 * p.rows * 4)));
        const uint32_t b_s = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)cb * (uint32_t)(16 * HW * 4)));
        if constexpr (QUAD) {
#pragma unroll
            for (int j = 0; j < NA; ++j) {
                const float4 v = buf_load4(rs_w, a_voff4, a_s + (uint32_t)(j * KPA) * (uint32_t)(p.rows * 4));
                ra[4 * j] = v.x, ra[4 * j + 1] = v.y, ra[4 * j + 2] = v.z, ra[4 * j + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < EA; ++j) ra[j] = buf_load(rs_w, a_voff, a_s + (uint32_t)(j * KSA) * (uint32_t)(p.rows * 4));
        }
        const int ih = ih0 + rr, iw = iw0 + ss;
        const bool ok = vm && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
        const uint32_t b_voff = ok ? (uint32_t)(pix_base + ih * p.W + iw) * 4u : kOobOffset;
#pragma unroll
        for (int j = 0; j < EB; ++j) rb[j] = buf_load(rs_src, b_voff, b_s + (uint32_t)(j * KSB) * (uint32_t)(HW * 4));
        // advance (cb, r, s): taps fastest, then channel block
        if (++s == p.S) {
            s = 0;
            if (++r == p.R) {
                r = 0;
                ++cb;
            }
        }
    };
    auto store_step = [&](int buf) {
        if constexpr (QUAD) {
#pragma unroll
            for (int j = 0; j < NA; ++j)
                a_st4[(buf * BK * LDA + j * KPA * LDA) / 4] = make_float4(ra[4 * j], ra[4 * j + 1], ra[4 * j + 2], ra[4 * j + 3]);
        } else {
#pragma unroll
            for (int j = 0; j < EA; ++j) a_st[buf * BK * LDA + j * KSA * LDA] = ra[j];
        }
#pragma unroll
        for (int j = 0; j < EB; ++j) b_st[buf * BK * LDB + j * KSB * LDB] = rb[j];
    };

    if (nsteps > 0) {
        load_step(step_begin);
        store_step(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nsteps; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nsteps;
        if (more) load_step(step_begin + kt + 1);
        const float* at = As + cur * BK * LDA + a_off;
        const float* bt = Bs + cur * BK * LDB + b_off;
        // operand fragments are read from LDS one k-pair ahead of the MFMAs that consume them
        float a[2][TM], b[2][TN];
        auto fetch_a = [&](float (&dst)[TM], const float* src) {
            if constexpr (PAIR_M) {
                const float2 v = *reinterpret_cast<const float2*>(src);
                dst[0] = v.x, dst[1] = v.y;
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i) dst[i] = src[i * 32];
            }
        };
        auto fetch_b = [&](float (&dst)[TN], const float* src) {
            if constexpr (PAIR_N) {
                const float2 v = *reinterpret_cast<const float2*>(src);
                dst[0] = v.x, dst[1] = v.y;
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j) dst[j] = src[j * 32];
            }
        };
        fetch_a(a[0], at);
        fetch_b(b[0], bt);
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const int c = (kk >> 1) & 1, nx = c ^ 1;
            if (kk + 2 < BK) {
                fetch_a(a[nx], at + (kk + 2) * LDA);
                fetch_b(b[nx], bt + (kk + 2) * LDB);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads above ahead of the MFMAs below
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            // the next step's tile goes to LDS half-way through this one: its write latency hides behind the
            // remaining MFMAs instead of standing between the last MFMA and the barrier
            if (kk == BK / 2 && more) {
                store_step(cur ^ 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    }

    if constexpr (SPLIT) {  // raw partial sums, tile-local [BM][BN]; conv_split_fixup_kernel finishes the tile
        float* pb = p.partial + (size_t)(tile_local * p.splits + split) * (BM * BN);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float* prow = pb + tile_row(i, v) * BN;
                if constexpr (PAIR_N) {
                    *reinterpret_cast<float2*>(prow + tile_col(0)) = make_float2(acc[i][0][v], acc[i][1][v]);
                } else {
#pragma unroll
                    for (int j = 0; j < TN; ++j) prow[tile_col(j)] = acc[i][j][v];
                }
            }
        return;
    }
    if constexpr (SPLIT) return;
    float* obase = p.out.base(0) + (size_t)group * p.out_gstride;
    if constexpr (PAIR_N) {
        const ConvOut::Col c0 = p.out.col(col0 + tile_col(0)), c1 = p.out.col(col0 + tile_col(1));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) p.out.put2(obase, row0 + tile_row(i, v), c0, c1, acc[i][0][v], acc[i][1][v]);
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const ConvOut::Col c = p.out.col(col0 + tile_col(j));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) p.out.put(obase, row0 + tile_row(i, v), c, acc[i][j][v]);
        }
    }
}

// Finishes the tiles whose reduction was split: adds the partial sums of a tile in split order (fixed:
// results do not depend on scheduling) and stores through the same epilogue as the unsplit kernel.
// kFixupChunks workgroups per tile, each a band of rows; lanes walk along pixels.
constexpr int kFixupChunks = 8;

template <int BM, int BN>
__global__ __launch_bounds__(kThreads) void conv_split_fixup_kernel(ConvFastParams p) {
    static_assert(BM % kFixupChunks == 0, "row bands");
    const int tile_local = blockIdx.x / kFixupChunks, chunk = blockIdx.x - tile_local * kFixupChunks;
    const int tile = p.tile_begin + tile_local;
    const int tile_n = tile / p.tiles_m, tile_m = tile - tile_n * p.tiles_m;
    const int row0 = tile_m * BM, col0 = tile_n * BN;
    const float* pb = p.partial + (size_t)tile_local * p.splits * (BM * BN);
    float* obase = p.out.base(0);
    const int col = threadIdx.x % BN;
    const ConvOut::Col c = p.out.col(col0 + col);
    const int r_end = (chunk + 1) * (BM / kFixupChunks);
    for (int row = chunk * (BM / kFixupChunks) + threadIdx.x / BN; row < r_end; row += kThreads / BN) {
        float acc = pb[row * BN + col];
#pragma unroll 4
        for (int s = 1; s < p.splits; ++s) acc += pb[(size_t)s * (BM * BN) + row * BN + col];
        p.out.put(obase, row0 + row, c, acc);
    }
}

}  // namespace vdnn

namespace vdnn {

// ---------------------------------------------------------------------------------------------
// Backward-filter fast path: dW[k][(tap, c)] = sum over pixels m = (n, p, q) of
// dY[n][k][p][q] * X[n][c][p*stride - pad + r][q*stride - pad + s].
// Columns are ordered tap-major and a column tile never straddles two taps (C is a multiple of the
// tile width), so the tap and the image-border test are the same for the whole workgroup and are
// evaluated once per K-step per thread.  Lanes walk along pixels (contiguous in NCHW).
// Partial sums of reduction split s go to ws[s][k][tap*C + c]; the launcher's reduction pass adds the splits
// in a fixed order and writes dW in [K][C][R][S] order.
// ---------------------------------------------------------------------------------------------
struct BwdFilterFastParams {
    const float* x;   // [N][C][H][W]
    const float* dy;  // [N][K][P][Q]
    float* ws;        // [splits][K][RS*C]
    uint32_t x_bytes, dy_bytes;
    int K, C, H, W, R, S, stride, pad, P, Q;
    int M;            // N*P*Q (reduction length)
    FastDiv fd_pq, fd_q;
    int tiles_m, tiles_n, splits, ksplit;
    // groups > 1: that many independent problems of the same shape in one launch; group g reads x + g * x_gstride and
    // dy + g * dy_gstride and writes ws + g * ws_gstride (strides in elements).  The grid is tiles * splits * groups.
    int groups = 1;
    size_t x_gstride = 0, dy_gstride = 0, ws_gstride = 0;
};

template <int BM, int BN, int WM, int WN, int BK, int TAPS = 1>
__global__ __launch_bounds__(kThreads) void conv_bwdf_fast_kernel(BwdFilterFastParams p) {
    constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "wave tiling");
    // A half-wave stores BK consecutive k (rows of LDS) x 32/BK consecutive columns: a row pitch of 32/BK words
    // (mod 32) spreads them over all 32 banks; fragment reads are 32 consecutive words and never conflict.
    constexpr int PAD = BK >= 32 ? 1 : 32 / BK;
    constexpr int LDA = BM + PAD, LDB = BN + PAD;
    constexpr int EA = BM * BK / kThreads, EB = BN * BK / kThreads;
    constexpr int RSTEP = kThreads / BK;  // 8 rows between a thread's elements
    extern __shared__ __align__(16) float smem[];
    float* As = smem;
    float* Bs = smem + 2 * BK * LDA;

    const int tid = threadIdx.x;
    const int tiles = p.tiles_m * p.tiles_n;
    int logical = xcd_remap(blockIdx.x, tiles * p.splits * p.groups);
    // the same for the whole workgroup; said explicitly so that the buffer resources below stay in scalar registers
    const int group = __builtin_amdgcn_readfirstlane(logical / (tiles * p.splits));
    logical -= group * (tiles * p.splits);
    const int split = logical / tiles;
    const int t2 = logical - split * tiles;
    const int tile_n = t2 / p.tiles_m, tile_m = t2 - tile_n * p.tiles_m;
    const int row0 = tile_m * BM, col0 = tile_n * BN;
    // TAPS == 1: the tile lies inside one tap.  TAPS > 1 (narrow layers, C == BN / TAPS): the tile covers TAPS whole
    // taps, CW = BN / TAPS channels each, so that a 64-channel layer still gets a wide tile.
    constexpr int CW = BN / TAPS;
    const int tap = col0 / p.C, c0 = col0 - tap * p.C;  // uniform
    int tr[TAPS], ts[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) { tr[t] = (tap + t) / p.S; ts[t] = (tap + t) - tr[t] * p.S; }
    const int kbeg = split * p.ksplit;
    const int kend = min(p.M, kbeg + p.ksplit);
    const int nk = (kend - kbeg + BK - 1) / BK;

    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.x + (size_t)group * p.x_gstride, p.x_bytes);
    const __amdgpu_buffer_rsrc_t rs_dy = make_rsrc(p.dy + (size_t)group * p.dy_gstride, p.dy_bytes);

    const int kk = tid % BK, r_first = tid / BK;
    const int PQ = p.P * p.Q, HW = p.H * p.W;
    const uint32_t a_rowpart = (uint32_t)(row0 + r_first) * (uint32_t)PQ;          // elements
    const uint32_t b_chpart = (uint32_t)(c0 + r_first) * (uint32_t)HW;

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int l32 = lane & 31, khalf = lane >> 5;
    // interleaved MFMA blocks and 8-byte fragment reads as in conv_fast_kernel (the row pitch must be even for those)
    constexpr bool PAIR_M = TM == 2 && LDA % 2 == 0, PAIR_N = TN == 2 && LDB % 2 == 0;
    const int a_off = khalf * LDA + wm * (TM * 32) + (PAIR_M ? 2 * l32 : l32);
    const int b_off = khalf * LDB + wn * (TN * 32) + (PAIR_N ? 2 * l32 : l32);
    auto tile_row = [&](int i, int v) {
        const int rr = 4 * khalf + 8 * (v / 4) + (v % 4);
        return wm * (TM * 32) + (PAIR_M ? 2 * rr + i : i * 32 + rr);
    };
    auto tile_col = [&](int j) { return wn * (TN * 32) + (PAIR_N ? 2 * l32 + j : j * 32 + l32); };
    float* a_st = As + kk * LDA + r_first;
    float* b_st = Bs + kk * LDB + r_first;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    float ra[EA], rb[EB];
    const bool full_rows = row0 + BM <= p.K;  // uniform
    auto load_step = [&](int k0) {
        const int m = k0 + kk;
        const bool vm = m < kend;
        const uint32_t mm = vm ? (uint32_t)m : 0u;
        const uint32_t n = fd_div(mm, p.fd_pq);
        const uint32_t pq = mm - n * (uint32_t)PQ;
        const uint32_t pp = fd_div(pq, p.fd_q);
        const uint32_t qq = pq - pp * (uint32_t)p.Q;
        uint32_t b_voff[TAPS];
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            const int ih = (int)pp * p.stride - p.pad + tr[t], iw = (int)qq * p.stride - p.pad + ts[t];
            const bool okb = vm && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
            b_voff[t] = okb ? (n * (uint32_t)p.C * (uint32_t)HW + (uint32_t)(ih * p.W + iw) + b_chpart) * 4u : kOobOffset;
        }
        // A: everything in the vector offset, so that rows past K (ragged last row tile) are either
        // another image's data (never stored) or out of range (0).
        const uint32_t a_base = vm ? (n * (uint32_t)p.K * (uint32_t)PQ + pq + a_rowpart) * 4u : kOobOffset;
        if (full_rows) {  // no row of the tile lies past K: the row step can ride in the scalar offset
#pragma unroll
            for (int j = 0; j < EA; ++j) ra[j] = buf_load(rs_dy, a_base, (uint32_t)(j * RSTEP) * (uint32_t)(PQ * 4));
        } else {
#pragma unroll
            for (int j = 0; j < EA; ++j) {
                const uint32_t v = vm ? a_base + (uint32_t)(j * RSTEP) * (uint32_t)(PQ * 4) : kOobOffset;
                ra[j] = buf_load(rs_dy, v, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < EB; ++j) {  // column r_first + j * RSTEP: tap (j * RSTEP) / CW, channel r_first + (j * RSTEP) % CW
            static_assert(TAPS == 1 || CW % RSTEP == 0, "a thread's columns must not straddle taps");
            rb[j] = buf_load(rs_x, b_voff[TAPS == 1 ? 0 : (j * RSTEP) / CW], (uint32_t)(TAPS == 1 ? j * RSTEP : (j * RSTEP) % CW) * (uint32_t)(HW * 4));
        }
    };
    auto store_step = [&](int buf) {
#pragma unroll
        for (int j = 0; j < EA; ++j) a_st[buf * BK * LDA + j * RSTEP] = ra[j];
#pragma unroll
        for (int j = 0; j < EB; ++j) b_st[buf * BK * LDB + j * RSTEP] = rb[j];
    };

    if (nk > 0) {
        load_step(kbeg);
        store_step(0);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) load_step(kbeg + (kt + 1) * BK);
        const float* at = As + cur * BK * LDA + a_off;
        const float* bt = Bs + cur * BK * LDB + b_off;
        float a[2][TM], b[2][TN];
        auto fetch_a = [&](float (&dst)[TM], const float* src) {
            if constexpr (PAIR_M) {
                const float2 v = *reinterpret_cast<const float2*>(src);
                dst[0] = v.x, dst[1] = v.y;
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i) dst[i] = src[i * 32];
            }
        };
        auto fetch_b = [&](float (&dst)[TN], const float* src) {
            if constexpr (PAIR_N) {
                const float2 v = *reinterpret_cast<const float2*>(src);
                dst[0] = v.x, dst[1] = v.y;
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j) dst[j] = src[j * 32];
            }
        };
        fetch_a(a[0], at);
        fetch_b(b[0], bt);
#pragma unroll
        for (int k2 = 0; k2 < BK; k2 += 2) {
            const int c = (k2 >> 1) & 1, nx = c ^ 1;
            if (k2 + 2 < BK) {
                fetch_a(a[nx], at + (k2 + 2) * LDA);
                fetch_b(b[nx], bt + (k2 + 2) * LDB);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the LDS reads above ahead of the MFMAs below
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[c][i], b[c][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (k2 == BK / 2 && more) {  // as in conv_fast_kernel
                store_step(cur ^ 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    }

    const int CRS = p.C * p.R * p.S;
    float* obase = p.ws + (size_t)group * p.ws_gstride + (size_t)split * p.K * CRS;
    // columns are < CRS (column tiles are never ragged here); CRS and a pair's first column are even
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row0 + tile_row(i, v);
            if (row >= p.K) continue;
            float* orow = obase + (size_t)row * CRS + col0;
            if constexpr (PAIR_N) {
                *reinterpret_cast<float2*>(orow + tile_col(0)) = make_float2(acc[i][0][v], acc[i][1][v]);
            } else {
#pragma unroll
                for (int j = 0; j < TN; ++j) orow[tile_col(j)] = acc[i][j][v];
            }
        }
}

}  // namespace vdnn
