// Linear projection y = x W^T on the bf16 matrix cores, with the K-vector
// norm of Eq. 4 (Sec. 3.2.2) produced in the epilogue: per row, the sum of
// squares of the rounded outputs of each group of 128 columns is written as
// one deterministic partial, so the selection pass never re-reads K.
//
// x [M,K] and W [N,K] are both contiguous along the contraction index, so the
// two MFMA operands are fetched the same way: a lane reads 8 consecutive
// k-values of one row.  The product is formed transposed (W tile as the A
// operand, x tile as the B operand): a lane then owns one output row m and
// 4-element runs of consecutive columns n, which gives 8-byte stores and
// in-lane row sums for the norm epilogue.
//
// Pipeline: k-steps of 64; two LDS stages; global -> registers -> LDS with the
// loads for step t+2 in flight while step t is multiplied; one barrier per
// k-step; MFMA fragments of the next 16-wide slice are read while the current
// slice is multiplied.  Workgroups are renumbered so that each XCD (own L2)
// works on a compact patch of output tiles.
#include "vitcop_internal.h"
#include "device_utils.h"

namespace vitcop {

constexpr int GM_THREADS = 256;
constexpr int GM_BK = 64;
constexpr int GM_LD = GM_BK + 8;     // bf16 per LDS row (144 B: conflict-free 16-byte reads)
constexpr int GM_PART = 128;         // columns per sum-of-squares partial
constexpr int GM_XCDS = 8;

template <int BM, int BN>
constexpr size_t gemm_lds_bytes() { return (size_t)2 * (BM + BN) * GM_LD * sizeof(uint16_t); }

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(GM_THREADS) void gemm_kernel(
    const uint16_t* __restrict__ x, int64_t x_stride, const uint16_t* __restrict__ w,
    uint16_t* __restrict__ y, int64_t y_stride, const uint16_t* __restrict__ res,
    int64_t res_stride, int M, int N, int K, float* __restrict__ sumsq_parts, int tiles_m,
    int tiles_n, int group_m) {
    static_assert(WAVES_M * WAVES_N == 4, "four wavefronts");
    constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N;
    constexpr int MI = TM / 32, NI = TN / 32;
    static_assert(TN == GM_PART, "one sum-of-squares partial per wavefront");
    constexpr int XCH = BM * GM_BK / 8 / GM_THREADS;   // 16-byte chunks per thread per stage
    constexpr int WCH = BN * GM_BK / 8 / GM_THREADS;
    constexpr int STAGE = (BM + BN) * GM_LD;           // elements per LDS stage

    extern __shared__ __attribute__((aligned(16))) uint16_t gemm_lds[];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wm = wv % WAVES_M, wn = wv / WAVES_M;

    // Workgroup -> tile.  Consecutive workgroup ids go to different XCDs, so id % 8 picks the
    // XCD and id / 8 the slot inside it; each XCD walks a contiguous range of a grouped
    // ordering (group_m tile rows by all tile columns, column-major inside the group).
    int tile_m, tile_n;
    {
        const int nt = tiles_m * tiles_n;
        const int pid = blockIdx.x;
        const int per = (nt + GM_XCDS - 1) / GM_XCDS;
        int lin = (pid % GM_XCDS) * per + pid / GM_XCDS;
        if (nt % GM_XCDS != 0) lin = pid;             // ragged: plain order
        const int width = group_m * tiles_n;
        const int grp = lin / width;
        const int first = grp * group_m;
        const int gsz = min(tiles_m - first, group_m);
        const int in = lin - grp * width;
        tile_m = first + in % gsz;
        tile_n = in / gsz;
    }
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    f32x16 acc[NI][MI];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < MI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // global -> register staging: chunk id -> (row = id / 8, 16-byte column = id % 8);
    // 32-bit element offsets from a base that advances with k (the host checks the range)
    // (unsigned byte offsets: base in scalar registers + one 32-bit register per chunk)
    const int srow = tid >> 3, scol = (tid & 7) * 8;      // chunk j sits 32*j rows further down
    unsigned xo[XCH], wo[WCH];
#pragma unroll
    for (int j = 0; j < XCH; ++j)
        xo[j] = 2u * (unsigned)(min(m0 + srow + 32 * j, M - 1) * (int)x_stride + scol);
#pragma unroll
    for (int j = 0; j < WCH; ++j)
        wo[j] = 2u * (unsigned)(min(n0 + srow + 32 * j, N - 1) * K + scol);
    // Two register staging sets; a tile is fetched two k-steps before it is written to LDS.
    // The 16-byte chunks of a tile (XCH of x, then WCH of W) are handled one quarter per
    // 16-wide slice, so the LDS writes and the global loads are spread over the whole k-step.
    constexpr int NCH = XCH + WCH, QCH = NCH / 4;
    static_assert(NCH % 4 == 0, "chunks split evenly over the four slices");
    u32x4 st[2][NCH];
    auto load_chunks = [&](int set, int k0, int c0, int c1) {
        const char* xb = reinterpret_cast<const char*>(x + k0);
        const char* wb = reinterpret_cast<const char*>(w + k0);
#pragma unroll
        for (int c = c0; c < c1; ++c)
            st[set][c] = c < XCH ? *reinterpret_cast<const u32x4*>(xb + xo[c < XCH ? c : 0])
                                 : *reinterpret_cast<const u32x4*>(wb + wo[c < XCH ? 0 : c - XCH]);
    };
    auto store_chunks = [&](int set, int stage, int c0, int c1) {
        uint16_t* Xs = gemm_lds + stage * STAGE + srow * GM_LD + scol;
        uint16_t* Ws = Xs + BM * GM_LD;
#pragma unroll
        for (int c = c0; c < c1; ++c) {
            if (c < XCH) *reinterpret_cast<u32x4*>(Xs + c * 32 * GM_LD) = st[set][c];
            else *reinterpret_cast<u32x4*>(Ws + (c - XCH) * 32 * GM_LD) = st[set][c];
        }
    };

    const int xoff = (wm * TM + l32) * GM_LD + g * 8;
    const int woff = BM * GM_LD + (wn * TN + l32) * GM_LD + g * 8;
    bf16x8 xf[2][MI], wf[2][NI];
    auto read_frags = [&](int buf, int stage, int kc) {
        const uint16_t* S = gemm_lds + stage * STAGE + kc * 16;
#pragma unroll
        for (int j = 0; j < MI; ++j)
            xf[buf][j] = *reinterpret_cast<const bf16x8*>(&S[xoff + j * 32 * GM_LD]);
#pragma unroll
        for (int i = 0; i < NI; ++i)
            wf[buf][i] = *reinterpret_cast<const bf16x8*>(&S[woff + i * 32 * GM_LD]);
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < MI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][i], xf[buf][j], acc[i][j], 0, 0, 0);
    };
    // scheduling hints: alternate one MFMA with `per` memory instructions of class `mask`
    // (0x100 LDS read, 0x200 LDS write, 0x020 global read), `n` times
#define VITCOP_INTERLEAVE(mask, per, n)                              \
    _Pragma("unroll") for (int q_ = 0; q_ < (n); ++q_) {             \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);           \
        __builtin_amdgcn_sched_group_barrier((mask), (per), 0);      \
    }
    constexpr int NFRAG = MI + NI, NMFMA = MI * NI;

    // Software pipeline over k-steps.  LDS stage s = t & 1 holds tile t; on entry to step t
    // register set s holds tile t+1 (its first quarter already in LDS and refilled with tile
    // t+3) and set s^1 holds tile t+2.  Step t, slice by slice (each slice: 16 MFMAs, the
    // fragment reads of the next slice, a quarter of the LDS writes and of the global loads):
    //   slices 0..2: quarters 1..3 of tile t+1 go from set s to stage s^1; each register is
    //                refilled with tile t+3 right after it is written
    //   barrier     (stage s^1 complete; nobody reads stage s any more: slice 3 was fetched)
    //   slice 3:     reads slice 0 of tile t+1 from stage s^1; quarter 0 of tile t+2 goes
    //                from set s^1 to stage s, refilled with tile t+4
    // Past the end the loads repeat the last tile and the extra LDS traffic is never consumed.
    const int nk = K / GM_BK;
    auto tile_k = [&](int tile) { return min(tile, nk - 1) * GM_BK; };
#define VITCOP_SLICE_HINTS()                                                         \
    if constexpr (NMFMA >= NFRAG + 2 * QCH) {                                        \
        VITCOP_INTERLEAVE(0x100, 1, NFRAG)                                           \
        VITCOP_INTERLEAVE(0x200, 1, QCH)                                             \
        VITCOP_INTERLEAVE(0x020, 1, QCH)                                             \
        __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG - 2 * QCH, 0);     \
    }
    auto step = [&](int t, int set) {
        const int s = set;             // == t & 1, kept a compile-time constant after inlining
        read_frags(1, s, 1);
        store_chunks(set, s ^ 1, QCH, 2 * QCH);
        load_chunks(set, tile_k(t + 3), QCH, 2 * QCH);
        multiply(0);
        VITCOP_SLICE_HINTS()

        read_frags(0, s, 2);
        store_chunks(set, s ^ 1, 2 * QCH, 3 * QCH);
        load_chunks(set, tile_k(t + 3), 2 * QCH, 3 * QCH);
        multiply(1);
        VITCOP_SLICE_HINTS()

        read_frags(1, s, 3);
        store_chunks(set, s ^ 1, 3 * QCH, NCH);
        load_chunks(set, tile_k(t + 3), 3 * QCH, NCH);
        multiply(0);
        VITCOP_SLICE_HINTS()

        __syncthreads();
        read_frags(0, s ^ 1, 0);
        store_chunks(set ^ 1, s, 0, QCH);
        load_chunks(set ^ 1, tile_k(t + 4), 0, QCH);
        multiply(1);
        VITCOP_SLICE_HINTS()
    };
    load_chunks(0, 0, 0, NCH);
    store_chunks(0, 0, 0, NCH);
    load_chunks(0, tile_k(1), 0, NCH);
    load_chunks(1, tile_k(2), 0, NCH);
    store_chunks(0, 1, 0, QCH);
    load_chunks(0, tile_k(3), 0, QCH);
    __syncthreads();
    read_frags(0, 0, 0);
    int t = 0;
    for (; t + 1 < nk; t += 2) {
        step(t, 0);
        step(t + 1, 1);
    }
    if (t < nk) step(t, 0);
#undef VITCOP_SLICE_HINTS
#undef VITCOP_INTERLEAVE

    // epilogue: lane owns row m = .. + l32 and columns n = .. + 8*(r/4) + 4*g + r%4
#pragma unroll
    for (int j = 0; j < MI; ++j) {
        const int m = m0 + wm * TM + j * 32 + l32;
        float ss = 0.f;
        if (m < M) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int n = n0 + wn * TN + i * 32 + 8 * r4 + 4 * g;
                    if (n < N) {                     // N % 4 == 0: the run of 4 is all in or all out
                        float c0 = acc[i][j][4 * r4], c1 = acc[i][j][4 * r4 + 1];
                        float c2 = acc[i][j][4 * r4 + 2], c3 = acc[i][j][4 * r4 + 3];
                        if (res) {
                            const uint2 rr = *reinterpret_cast<const uint2*>(res + (int64_t)m * res_stride + n);
                            c0 += bf16_lo(rr.x); c1 += bf16_hi(rr.x);
                            c2 += bf16_lo(rr.y); c3 += bf16_hi(rr.y);
                        }
                        uint2 pk;
                        pk.x = pack_bf16(c0, c1);
                        pk.y = pack_bf16(c2, c3);
                        *reinterpret_cast<uint2*>(y + (int64_t)m * y_stride + n) = pk;
                        if (sumsq_parts) {
                            float a;
                            a = bf16_lo(pk.x); ss = fmaf(a, a, ss);
                            a = bf16_hi(pk.x); ss = fmaf(a, a, ss);
                            a = bf16_lo(pk.y); ss = fmaf(a, a, ss);
                            a = bf16_hi(pk.y); ss = fmaf(a, a, ss);
                        }
                    }
                }
        }
        if (sumsq_parts) {
            ss += __shfl_xor(ss, 32, 64);
            const int part = (n0 + wn * TN) / GM_PART;
            if (g == 0 && m < M && n0 + wn * TN < N) sumsq_parts[(int64_t)part * M + m] = ss;
        }
    }
}

int gemm_sumsq_parts(int N) { return (N + GM_PART - 1) / GM_PART; }

template <int BM, int BN, int WAVES_M, int WAVES_N>
static int launch_gemm_cfg(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y,
                           int64_t y_stride, const uint16_t* res, int64_t res_stride, int M, int N,
                           int K, float* sumsq_parts, hipStream_t s) {
    auto kern = gemm_kernel<BM, BN, WAVES_M, WAVES_N>;
    constexpr size_t lds = gemm_lds_bytes<BM, BN>();
    static bool attr_set = false;        // per kernel instantiation; setting it twice is harmless
    if (!attr_set) {
        int rc = hip_status(hipFuncSetAttribute((const void*)kern,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                            "hipFuncSetAttribute(gemm)");
        if (rc) return rc;
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    // tile rows per group: a patch of about 32 tiles (one XCD's worth of workgroups) near square
    int group_m = 1;
    while (group_m * 2 <= tiles_m && group_m * group_m * 2 <= 32) group_m *= 2;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(GM_THREADS), lds, s, x, x_stride, w, y,
                       y_stride, res, res_stride, M, N, K, sumsq_parts, tiles_m, tiles_n, group_m);
    return launch_status("gemm");
}

int launch_gemm(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y,
                int64_t y_stride, const uint16_t* res, int64_t res_stride, int M, int N,
                int K, float* sumsq_parts, hipStream_t s) {
    if (M == 0 || N == 0) return VITCOP_OK;
    // large problems: 256x256 tiles (each wavefront 128x128); otherwise 128x128 tiles
    const long big_tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
    if (big_tiles >= 192)
        return launch_gemm_cfg<256, 256, 2, 2>(x, x_stride, w, y, y_stride, res, res_stride, M, N, K,
                                               sumsq_parts, s);
    return launch_gemm_cfg<128, 128, 4, 1>(x, x_stride, w, y, y_stride, res, res_stride, M, N, K,
                                           sumsq_parts, s);
}

}  // namespace vitcop
