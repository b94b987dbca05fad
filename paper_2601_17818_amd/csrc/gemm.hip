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
// Pipeline: k-steps of 32 held in a ring of four LDS slabs that are filled by direct
// global -> LDS loads (no register staging), three k-steps in flight; one barrier per
// k-step; MFMA fragments of the next 16-wide slice are read while the current
// slice is multiplied.  Workgroups are renumbered so that each XCD (own L2)
// works on a compact patch of output tiles.
#include <atomic>
#include "vitcop_internal.h"
#include "device_utils.h"

namespace vitcop {

constexpr int GM_THREADS = 256;
constexpr int GM_SLABS = 4;          // ring of k-slabs in LDS: three k-steps of loads in flight (k-steps of 32)
constexpr int GM_PART = 128;         // columns per sum-of-squares partial
constexpr int GM_XCDS = 8;

// LDS: the slab ring, reused by the epilogue as one staging region per wavefront of
// (BM / WAVES_M) rows of (BN / WAVES_N) bf16 + 16 bytes of padding.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NS = GM_SLABS>
constexpr size_t gemm_lds_bytes() {
    constexpr size_t ring = (size_t)NS * (BM + BN) * BK * 2;
    constexpr size_t stage = (size_t)4 * (BM / WAVES_M) * ((BN / WAVES_N) * 2 + 16);
    return ring > stage ? ring : stage;
}

// A slab row holds BK bf16 (64 or 128 bytes, unpadded because direct loads write 1 KiB runs).
// 16-byte chunk c of row r lives at chunk position c ^ swz(r), which makes the MFMA fragment
// reads (32 consecutive rows, same chunk) bank-conflict free: LDS serves a 16-byte read 16 lanes at a
// time, so 16 consecutive rows must fall on the 16 different 16-byte units of a 256-byte bank row.  With
// 64-byte rows the unit is 4*(r & 3) + position, so the position must differ among r, r+4, r+8, r+12;
// with 128-byte rows it is 8*(r & 1) + position, so it must differ among the eight rows of equal parity.
template <int BK>
__device__ __forceinline__ int gm_swz(int row) {
    return BK == 32 ? (row >> 2) & 3 : (row >> 1) & 7;
}

// y = x W^T (+ residual).  With w2 != nullptr the columns [n_split, N) come from a second weight
// matrix and go to a second output (two projections of the same input in one launch).
// EPI selects the epilogue: GM_EPI_BF16 the projection described above; GM_EPI_DIST writes,
// in fp32, the Euclidean distance between row m of x and row n of w from their inner product
// and the two squared row norms: dist[m,n] = sqrt(max(0, xsq[m] + wsq[n] - 2 <x_m, w_n>)).
// GM_EPI_PART is split-K: blockIdx.y = split, which multiplies its share of the k-steps and writes the
// raw fp32 accumulators to dist[split][m][n] (row stride dist_stride, slices dist_batch apart) for a
// reduction kernel to add up.
// GM_EPI_GATED is the MLP's first half in one launch: a tile's first BN/2 columns are rows of w (gate), its
// last BN/2 the same rows of w2 (up); N counts the columns of each; the epilogue rounds both to bf16 as the
// two separate projections would, and stores y[m,n] = silu(gate[m,n]) * up[m,n] (WAVES_N == 2: the gate
// columns of a tile belong to the wavefronts with wn = 0, the up columns to wn = 1).
constexpr int GM_EPI_BF16 = 0, GM_EPI_DIST = 1, GM_EPI_PART = 2, GM_EPI_GATED = 3;

// BK, NS: k-step and slabs in the ring.  With k-steps of 64 a slab row is a whole 128-byte line, so one direct
// load moves 8 whole lines where k-steps of 32 move 16 half lines (and fetch every line twice, one k-step
// apart): the CU's load path, which is what bounds the tiles of 128 and 192 columns, carries twice the useful
// bytes.  Tiles whose three 64-wide slabs do not fit in LDS (256 x 256, 192 x 256) stay at 32 with four slabs;
// with two slabs of 64 they were slower.
template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int EPI = GM_EPI_BF16, int NS = GM_SLABS>
__global__ __launch_bounds__(GM_THREADS) void gemm_kernel(
    const uint16_t* __restrict__ x, int64_t x_stride, const uint16_t* __restrict__ w,
    uint16_t* __restrict__ y, int64_t y_stride, const uint16_t* __restrict__ res,
    int64_t res_stride, int M, int N, int K, float* __restrict__ sumsq_parts, int tiles_m,
    int tiles_n, int group_m, const uint16_t* __restrict__ w2, uint16_t* __restrict__ y2,
    int n_split, int64_t w_stride, const float* __restrict__ xsq, const float* __restrict__ wsq,
    float* __restrict__ dist, int64_t dist_stride, int64_t x_batch, int64_t sq_batch,
    int64_t dist_batch) {
    static_assert(WAVES_M * WAVES_N == 4, "four wavefronts");
    static_assert(BK == 32 || BK == 64, "slab rows of 64 or 128 bytes");
    constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int ROWB = BK * 2;                         // bytes per slab row
    constexpr int CHUNKS = BK / 8;                       // 16-byte chunks per row
    constexpr int ROWS_PER_LOAD = 64 / CHUNKS;           // rows covered by one 1 KiB direct load
    constexpr int KC = BK / 16;                          // 16-wide MFMA slices per k-step
    constexpr int SLAB = (BM + BN) * ROWB;               // bytes per slab
    constexpr int NDMA = SLAB / 1024 / 4;                // direct loads per wavefront per slab
    static_assert(SLAB % 4096 == 0 && (BM * ROWB) % 1024 == 0, "slab splits evenly over loads");

    extern __shared__ __attribute__((aligned(1024))) char gemm_lds[];
    if constexpr (EPI == GM_EPI_PART) dist += blockIdx.y * dist_batch;
    if constexpr (EPI == GM_EPI_DIST) {      // blockIdx.y = image: x and w are the same feature matrix
        x += blockIdx.y * x_batch;
        w += blockIdx.y * x_batch;
        xsq += blockIdx.y * sq_batch;
        wsq += blockIdx.y * sq_batch;
        dist += blockIdx.y * dist_batch;
    }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront index, kept scalar
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
    const int m0 = tile_m * BM;
    int n0 = tile_n * (EPI == GM_EPI_GATED ? BN / 2 : BN);
    if constexpr (EPI == GM_EPI_GATED) {
        static_assert(EPI != GM_EPI_GATED || WAVES_N == 2, "gate and up halves go to the two wavefront columns");
    } else if (w2 != nullptr && n0 >= n_split) {         // second projection (uniform per workgroup)
        w = w2;
        y = y2;
        n0 -= n_split;
        N -= n_split;
        if constexpr (EPI == GM_EPI_PART) dist += n_split;       // the partials keep the launch's column index
    } else if (w2 != nullptr) {
        N = n_split;
    }

    f32x16 acc[NI][MI];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < MI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Direct global -> LDS loads.  Load q of wavefront wv fills slab bytes [(wv*NDMA+q)*1024, +1024):
    // ROWS_PER_LOAD rows; lane L lands at row L / CHUNKS, chunk position L % CHUNKS, so it must
    // fetch the chunk that the swizzle assigns to that position.  Rows [0,BM) are x, then W.
    unsigned goff[NDMA];             // byte offset of this lane's chunk from x (or W) at k = 0
#pragma unroll
    for (int q = 0; q < NDMA; ++q) {
        const int row = (wv * NDMA + q) * ROWS_PER_LOAD + lane / CHUNKS;        // slab row
        const int chunk = (lane % CHUNKS) ^ gm_swz<BK>(row);
        if (row < BM)
            goff[q] = 2u * (unsigned)(min(m0 + row, M - 1) * (int)x_stride + chunk * 8);
        else if (EPI == GM_EPI_GATED)     // slab rows [BM, BM + BN/2): gate rows n0.., then the same rows of up
            goff[q] = 2u * (unsigned)(min(n0 + (row - BM) % (BN / 2), N - 1) * (int)w_stride + chunk * 8);
        else
            goff[q] = 2u * (unsigned)(min(n0 + row - BM, N - 1) * (int)w_stride + chunk * 8);
    }
    auto issue_loads = [&](int slab, int k0, int part = 0, int parts = 1) {
        const char* xb = reinterpret_cast<const char*>(x + k0);
        const char* wb = reinterpret_cast<const char*>(w + k0);
        const char* ub = reinterpret_cast<const char*>((EPI == GM_EPI_GATED ? w2 : w) + k0);
#pragma unroll
        for (int q = 0; q < NDMA; ++q) {
            if (q * parts / NDMA != part) continue;
            const bool is_x = (wv * NDMA + q) * ROWS_PER_LOAD < BM;            // wave-uniform
            const bool is_up = EPI == GM_EPI_GATED && (wv * NDMA + q) * ROWS_PER_LOAD >= BM + BN / 2;
            const char* src = (is_x ? xb : is_up ? ub : wb) + goff[q];
            char* dst = gemm_lds + slab * SLAB + (wv * NDMA + q) * 1024;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)src,
                (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        }
    };

    // MFMA fragments: lane (l32, g) reads 8 consecutive k of row l32: chunk 2*kc + g
    int xrow[MI], wrow[NI];
#pragma unroll
    for (int j = 0; j < MI; ++j) xrow[j] = wm * TM + j * 32 + l32;
#pragma unroll
    for (int i = 0; i < NI; ++i) wrow[i] = BM + wn * TN + i * 32 + l32;
    bf16x8 xf[2][MI], wf[2][NI];
    auto read_frags = [&](int buf, int slab, int kc) {
        const char* S = gemm_lds + slab * SLAB;
#pragma unroll
        for (int j = 0; j < MI; ++j)
            xf[buf][j] = *reinterpret_cast<const bf16x8*>(
                S + xrow[j] * ROWB + (((2 * kc + g) ^ gm_swz<BK>(xrow[j])) << 4));
#pragma unroll
        for (int i = 0; i < NI; ++i)
            wf[buf][i] = *reinterpret_cast<const bf16x8*>(
                S + wrow[i] * ROWB + (((2 * kc + g) ^ gm_swz<BK>(wrow[i])) << 4));
    };
    auto multiply = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < MI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][i], xf[buf][j], acc[i][j], 0, 0, 0);
    };
    // scheduling hints: alternate one MFMA with one memory instruction of class `mask`, n times
    // (0x100 LDS read, 0x020 global read)
#define VITCOP_INTERLEAVE(mask, n)                                   \
    _Pragma("unroll") for (int q_ = 0; q_ < (n); ++q_) {             \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);           \
        __builtin_amdgcn_sched_group_barrier((mask), 1, 0);          \
    }
    constexpr int NFRAG = MI + NI, NMFMA = MI * NI;
    // A step's loads go out in equal shares, one per slice, the last share after the barrier (into the same
    // slab, free since the barrier of the step before): issued together, one CU's 4 x NDMA loads saturate its
    // load unit for the whole first slice, and a wavefront stuck on issuing one cannot issue MFMAs meanwhile
    // (8 % fewer cycles on the 256 x 256 tile, 3-6 % more throughput on the smaller ones).  SPLIT: the form
    // with two slices and enough MFMAs to pair every fragment read and load with one (scheduling hints).
    constexpr bool SPLIT = KC == 2 && NDMA % 2 == 0 && NMFMA >= NFRAG + NDMA;
    constexpr bool SPREAD = !SPLIT && NDMA >= KC;
    constexpr int LAST_PART = NDMA - ((KC - 1) * NDMA + KC - 1) / KC;      // loads issued after the barrier

    // Pipeline over k-steps of BK.  Slab t % NS holds k-step t; the loads of k-step t+NS-1 are
    // issued during step t into the slab that step t-1 used (every wavefront left it before
    // the barrier of step t-1).  Step t, slice by slice (a slice = 16 of k):
    //   slice 0: multiply; read the fragments of slice 1; issue the loads of step t+NS-1 (or their first half)
    //   slices 1 .. KC-2: multiply; read the fragments of the next slice
    //   wait until this wavefront's loads of step t+1 have landed (NS-2 younger steps may
    //   still be in flight); barrier
    //   slice KC-1: multiply; read the fragments of slice 0 of step t+1 (and issue the second half)
    // Past the end the loads repeat the last k-step into slabs nobody reads again.
    int nk = K / BK, k_lo = 0;
    if constexpr (EPI == GM_EPI_PART) {      // this split's k-steps: [k_lo, k_lo + nk), never empty
        const int all = nk;
        k_lo = (int)((int64_t)all * blockIdx.y / gridDim.y);
        nk = (int)((int64_t)all * (blockIdx.y + 1) / gridDim.y) - k_lo;
    }
    auto k_of = [&](int step) { return (k_lo + min(step, nk - 1)) * BK; };
    auto step = [&](int t, int slab) {
#pragma unroll
        for (int kc = 0; kc < KC - 1; ++kc) {
            read_frags((kc + 1) & 1, slab, kc + 1);
            if constexpr (SPREAD) {
                issue_loads((slab + NS - 1) % NS, k_of(t + NS - 1), kc, KC);
            } else if (kc == 0) {
                if constexpr (SPLIT) issue_loads((slab + NS - 1) % NS, k_of(t + NS - 1), 0, 2);
                else issue_loads((slab + NS - 1) % NS, k_of(t + NS - 1));
            }
            multiply(kc & 1);
            if constexpr (NMFMA >= NFRAG + NDMA) {
                VITCOP_INTERLEAVE(0x100, NFRAG)
                if (kc == 0) {
                    VITCOP_INTERLEAVE(0x020, (SPLIT ? NDMA / 2 : NDMA))
                    __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG - (SPLIT ? NDMA / 2 : NDMA), 0);
                } else {
                    __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, 0);
                }
            }
        }
        // (a plain s_barrier: __syncthreads would also drain the two younger steps' loads)
        // (younger loads that may stay in flight: the steps t+2 .. t+NS-2 and what this step has issued so far)
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NDMA - (SPLIT ? NDMA / 2 : SPREAD ? LAST_PART : 0)) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        read_frags(KC & 1, (slab + 1) % NS, 0);
        // second half of this step's loads: same slab (free since the barrier of the step before)
        if constexpr (SPLIT) issue_loads((slab + NS - 1) % NS, k_of(t + NS - 1), 1, 2);
        if constexpr (SPREAD) issue_loads((slab + NS - 1) % NS, k_of(t + NS - 1), KC - 1, KC);
        multiply((KC - 1) & 1);
        if constexpr (NMFMA >= NFRAG) {
            VITCOP_INTERLEAVE(0x100, NFRAG)
            if constexpr (SPLIT) {
                VITCOP_INTERLEAVE(0x020, NDMA / 2)
                __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG - NDMA / 2, 0);
            } else {
                __builtin_amdgcn_sched_group_barrier(0x008, NMFMA - NFRAG, 0);
            }
        }
    };
    static_assert(NS >= 3 && (NS - 2) * NDMA <= 63, "the wait counter holds 63 loads");
#pragma unroll
    for (int i = 0; i < NS - 1; ++i) issue_loads(i, k_of(i));
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NDMA) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    read_frags(0, 0, 0);
    int t = 0;
    for (; t + NS - 1 < nk; t += NS) {
#pragma unroll
        for (int i = 0; i < NS; ++i) step(t + i, i);
    }
#pragma unroll
    for (int i = 0; i < NS - 1; ++i)
        if (t + i < nk) step(t + i, i);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // no load may outlive the workgroup's LDS
#undef VITCOP_INTERLEAVE

    if constexpr (EPI == GM_EPI_PART) {
        // lane owns row m = .. + l32 and the 4-element column runs n = .. + 8*(r/4) + 4*g + r%4
#pragma unroll
        for (int j = 0; j < MI; ++j) {
            const int m = m0 + wm * TM + j * 32 + l32;
            if (m >= M) continue;
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int n = n0 + wn * TN + i * 32 + 8 * r4 + 4 * g;
                    if (n >= N) continue;            // N % 4 == 0: the run of 4 is all in or all out
                    float4 o;
                    o.x = acc[i][j][4 * r4];
                    o.y = acc[i][j][4 * r4 + 1];
                    o.z = acc[i][j][4 * r4 + 2];
                    o.w = acc[i][j][4 * r4 + 3];
                    *reinterpret_cast<float4*>(dist + (int64_t)m * dist_stride + n) = o;
                }
        }
        return;
    }
    if constexpr (EPI == GM_EPI_DIST) {
        // lane owns row m = .. + l32 and the 4-element column runs n = .. + 8*(r/4) + 4*g + r%4
#pragma unroll
        for (int j = 0; j < MI; ++j) {
            const int m = m0 + wm * TM + j * 32 + l32;
            if (m >= M) continue;
            const float sm = xsq[m];
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int n = n0 + wn * TN + i * 32 + 8 * r4 + 4 * g;
                    if (n >= N) continue;
                    // wsq and the rows of dist are padded to a multiple of 4 entries, so the run
                    // of 4 may be read and written whole even when N cuts it
                    const float4 sn = *reinterpret_cast<const float4*>(wsq + n);
                    float4 o;
                    o.x = __builtin_sqrtf(fmaxf(0.f, fmaf(-2.f, acc[i][j][4 * r4], sm + sn.x)));
                    o.y = __builtin_sqrtf(fmaxf(0.f, fmaf(-2.f, acc[i][j][4 * r4 + 1], sm + sn.y)));
                    o.z = __builtin_sqrtf(fmaxf(0.f, fmaf(-2.f, acc[i][j][4 * r4 + 2], sm + sn.z)));
                    o.w = __builtin_sqrtf(fmaxf(0.f, fmaf(-2.f, acc[i][j][4 * r4 + 3], sm + sn.w)));
                    *reinterpret_cast<float4*>(dist + (int64_t)m * dist_stride + n) = o;
                }
        }
        return;
    }
    // Epilogue.  In the accumulators a lane owns row m = .. + l32 and 4-element runs of columns
    // n = .. + 8*(r/4) + 4*g + r%4: stored directly, every store instruction would touch 32
    // rows with 16 bytes each, and the L2 request rate of all CUs finishing a round together
    // becomes the bottleneck.  So the rounded tile goes through LDS (the slab ring is free now):
    // each wavefront stages its own TM x TN block, rows padded by 16 bytes, and writes it out
    // with 16 bytes per lane, consecutive lanes along a row.  The residual is added and the
    // norm partial is formed on the way in, in the accumulator layout.
    constexpr int STAGE_ROW = TN * 2 + 16;                // bytes; the pad spreads the rows over the banks
    __builtin_amdgcn_s_barrier();                         // every wavefront is done reading the slabs
    char* stage = gemm_lds + wv * (TM * STAGE_ROW);
#pragma unroll
    for (int j = 0; j < MI; ++j) {
        const int m = m0 + wm * TM + j * 32 + l32;
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int n = n0 + wn * TN + i * 32 + 8 * r4 + 4 * g;
                float c0 = acc[i][j][4 * r4], c1 = acc[i][j][4 * r4 + 1];
                float c2 = acc[i][j][4 * r4 + 2], c3 = acc[i][j][4 * r4 + 3];
                if (res) {
                    if (m < M && n < N) {            // N % 4 == 0: the run of 4 is all in or all out
                        const uint2 rr = *reinterpret_cast<const uint2*>(res + (int64_t)m * res_stride + n);
                        c0 += bf16_lo(rr.x); c1 += bf16_hi(rr.x);
                        c2 += bf16_lo(rr.y); c3 += bf16_hi(rr.y);
                    }
                }
                uint2 pk;
                pk.x = pack_bf16(c0, c1);
                pk.y = pack_bf16(c2, c3);
                *reinterpret_cast<uint2*>(stage + (j * 32 + l32) * STAGE_ROW + (i * 32 + 8 * r4 + 4 * g) * 2) = pk;
                if constexpr (TN == GM_PART) {
                    if (sumsq_parts && n < N) {      // squares of the ROUNDED outputs, two per instruction
                        const bf16x2 lo = __builtin_bit_cast(bf16x2, pk.x), hi = __builtin_bit_cast(bf16x2, pk.y);
                        ss = __builtin_amdgcn_fdot2_f32_bf16(lo, lo, ss, false);
                        ss = __builtin_amdgcn_fdot2_f32_bf16(hi, hi, ss, false);
                    }
                }
            }
        if constexpr (TN == GM_PART) {           // one partial per wavefront; other layouts never get sumsq_parts
            if (sumsq_parts) {
                ss += __shfl_xor(ss, 32, 64);
                const int part = (n0 + wn * TN) / GM_PART;
                if (g == 0 && m < M && n0 + wn * TN < N) sumsq_parts[(int64_t)part * M + m] = ss;
            }
        }
    }
    if constexpr (EPI == GM_EPI_GATED) {
        // gate block of these rows: staged by wavefront (wm, 0); up block: by (wm, 1).  Each of the two takes
        // half of the block's columns: 16-byte chunks of gate and up in, one chunk of silu(gate) * up out.
        static_assert((BM * ROWB) % (ROWS_PER_LOAD * ROWB) == 0 && (BN / 2) % ROWS_PER_LOAD == 0, "whole loads per half");
        __builtin_amdgcn_s_waitcnt(0xC07F);               // lgkmcnt(0): this wavefront's staging writes are done
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        const char* gate_stage = gemm_lds + wm * (TM * STAGE_ROW);
        const char* up_stage = gemm_lds + (wm + WAVES_M) * (TM * STAGE_ROW);
        constexpr int HALF_LANES = TN / 16;               // 16-byte chunks per half row
        constexpr int ROWS_PER_PASS = 64 / HALF_LANES;    // (96-column blocks: 10 rows, the last 4 lanes idle)
        const int hrow = lane / HALF_LANES, hchunk = lane % HALF_LANES + wn * HALF_LANES;
        const int nn = n0 + hchunk * 8;
        if (nn < N && hrow < ROWS_PER_PASS) {             // N % 8 == 0: the chunk is all in or all out
#pragma unroll
            for (int r0 = 0; r0 < TM; r0 += ROWS_PER_PASS) {
                const int row = r0 + hrow;
                if (TM % ROWS_PER_PASS != 0 && row >= TM) break;
                const int m = m0 + wm * TM + row;
                const u32x4 gv = *reinterpret_cast<const u32x4*>(gate_stage + row * STAGE_ROW + hchunk * 16);
                const u32x4 uv = *reinterpret_cast<const u32x4*>(up_stage + row * STAGE_ROW + hchunk * 16);
                u32x4 ov;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float g0 = bf16_lo(gv[e]), g1 = bf16_hi(gv[e]);
                    const float s0 = g0 / (1.0f + __expf(-g0)), s1 = g1 / (1.0f + __expf(-g1));
                    ov[e] = pack_bf16(s0 * bf16_lo(uv[e]), s1 * bf16_hi(uv[e]));
                }
                if (m < M) *reinterpret_cast<u32x4*>(y + (int64_t)m * y_stride + nn) = ov;
            }
        }
        return;
    }
    // (a wavefront reads back only what it wrote itself: no barrier, the LDS counter suffices)
    constexpr int LANES_PER_ROW = TN / 8;                 // 16-byte chunks per staged row
    constexpr int ROWS_PER_STORE = 64 / LANES_PER_ROW;
    const int srow = lane / LANES_PER_ROW, schunk = lane % LANES_PER_ROW;
    const int n = n0 + wn * TN + schunk * 8;
    if (n < N) {                                          // N % 8 == 0: the chunk is all in or all out
#pragma unroll
        for (int r0 = 0; r0 < TM; r0 += ROWS_PER_STORE) {
            const int row = r0 + srow;
            const int m = m0 + wm * TM + row;
            const u32x4 val = *reinterpret_cast<const u32x4*>(stage + row * STAGE_ROW + schunk * 16);
            if (m < M) *reinterpret_cast<u32x4*>(y + (int64_t)m * y_stride + n) = val;
        }
    }
}

int gemm_sumsq_parts(int N) { return (N + GM_PART - 1) / GM_PART; }

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int EPI = GM_EPI_BF16, int NS = GM_SLABS>
static int launch_gemm_cfg(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y,
                           int64_t y_stride, const uint16_t* res, int64_t res_stride, int M, int N,
                           int K, float* sumsq_parts, const uint16_t* w2, uint16_t* y2, int n_split,
                           hipStream_t s, int64_t w_stride = 0, const float* xsq = nullptr,
                           const float* wsq = nullptr, float* dist = nullptr, int64_t dist_stride = 0,
                           int batch = 1, int64_t x_batch = 0, int64_t sq_batch = 0, int64_t dist_batch = 0) {
    if (w_stride == 0) w_stride = K;
    auto kern = gemm_kernel<BM, BN, WAVES_M, WAVES_N, BK, EPI, NS>;
    constexpr size_t lds = gemm_lds_bytes<BM, BN, WAVES_M, WAVES_N, BK, NS>();
    static_assert(lds <= 160 * 1024, "LDS of a CU");
    static std::atomic<bool> attr_set{false};   // per kernel instantiation; a second thread repeating the call is harmless
    if (!attr_set.load(std::memory_order_acquire)) {
        int rc = hip_status(hipFuncSetAttribute((const void*)kern,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                            "hipFuncSetAttribute(gemm)");
        if (rc) return rc;
        attr_set.store(true, std::memory_order_release);
    }
    const int tiles_m = (M + BM - 1) / BM;
    const int tiles_n = EPI == GM_EPI_GATED ? (N + BN / 2 - 1) / (BN / 2) : (N + BN - 1) / BN;
    // tile rows per group: a patch of about 32 tiles (one XCD's worth of workgroups) near square
    int group_m = 1;
    while (group_m * 2 <= tiles_m && group_m * group_m * 2 <= 32) group_m *= 2;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n, batch), dim3(GM_THREADS), lds, s, x, x_stride, w, y,
                       y_stride, res, res_stride, M, N, K, sumsq_parts, tiles_m, tiles_n, group_m, w2,
                       y2, n_split, w_stride, xsq, wsq, dist, dist_stride, x_batch, sq_batch, dist_batch);
    return launch_status("gemm");
}

// The k-step of a launch: 64 where three (or four) slabs of that width fit in LDS and K allows it, else 32.
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, typename... Args>
static int launch_gemm_k(int K, Args... args) {
    constexpr size_t slab64 = (size_t)(BM + BN) * 128;
    if constexpr (3 * slab64 <= 160 * 1024) {
        constexpr int NS = 4 * slab64 <= 160 * 1024 ? 4 : 3;
        if (K % 64 == 0) return launch_gemm_cfg<BM, BN, WAVES_M, WAVES_N, 64, EPI, NS>(args...);
    }
    return launch_gemm_cfg<BM, BN, WAVES_M, WAVES_N, 32, EPI>(args...);
}

// Tile shapes.  The wavefront tile sets the LDS bytes read per MFMA, so big tiles are the
// efficient ones; smaller ones exist to fill all 256 CUs when there are few rows.  `rate` is
// the measured throughput of a CU on that shape relative to 256x256 (K = 4096, full rounds).
struct TileShape {
    int bm, bn;
    float rate;
    bool sumsq;        // wavefront tile is 128 columns wide: can emit the norm partials
};
enum TileId { T256x256, T192x256, T256x128, T192x128, T128x128, T128x128R, T128x32, T192x192G, T_COUNT };
static const TileShape kTiles[T_COUNT] = {
    {256, 256, 1.00f, true},  {192, 256, 0.90f, true},  {256, 128, 0.88f, false}, {192, 128, 0.89f, false},
    {128, 128, 0.76f, false}, {128, 128, 0.74f, true},  {128, 32, 0.0f, false},
    {192, 192, 0.88f, false},     // gate/up launches only (96 gate + 96 up columns): its epilogue exists in that form alone
};

// Estimated time of the launch in units of (one 256x256 tile at full rate): rounds over the
// 256 CUs times the time of one tile.
static float tile_cost(const TileShape& t, int M, int N) {
    const long tiles = (long)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
    const long rounds = (tiles + 255) / 256;
    return (float)rounds * (float)(t.bm * t.bn) / (65536.0f * t.rate);
}

// Few rows and no norm output: the weight matrix dominates the traffic and one CU cannot pull
// its share fast enough, so the columns are cut into 32-wide tiles to put every CU to work.
static bool prefer_skinny_tiles(int M, int N, int K) {
    const long mid = (long)((M + 127) / 128) * ((N + 127) / 128);
    return mid <= 64 && K % 64 == 0 && N % 32 == 0;
}

static TileId choose_tile(int M, int N, int K, bool need_sumsq, int align_n) {
    if (!need_sumsq && prefer_skinny_tiles(M, N, K)) return T128x32;
    TileId best = need_sumsq ? T128x128R : T128x128;
    float best_cost = tile_cost(kTiles[best], M, N);
    for (int i = 0; i < T128x32; ++i) {
        const TileShape& t = kTiles[i];
        if (need_sumsq && !t.sumsq) continue;
        if (align_n % t.bn != 0) continue;           // a tile must not straddle the two outputs of a pair
        const float c = tile_cost(t, M, N);
        if (c < best_cost) {
            best_cost = c;
            best = (TileId)i;
        }
    }
    return best;
}

// A launch whose tiles overflow whole rounds over the 256 CUs by a few (640 rows x 22016 columns: 3 x 86 =
// 258 tiles of 256 x 256) would spend a whole extra round on them.  Then only the leading columns, as many
// column tiles as fill the whole rounds, go out on the big tiles, and the few trailing columns follow as a
// launch of their own on the few-row / split-K path, which spreads them over the chip.  Returns the number
// of leading columns (N: no cut) and, in `id`, the tile shape for them.  A small tail (at most 64 tiles'
// worth) is priced at 0.3 of a 256 x 256 tile time (its launch and its reduction); a larger one goes out on
// whichever tile shape suits its own size and is priced as that launch plus the boundary between the two
// (5120 x 4096: 320 tiles of 256 x 256 are 1.25 rounds; 240 of them and then 160 tiles of 256 x 128 are
// one round each at their rates, 1.57 tile times instead of 2).
constexpr int GM_TAIL_MAX_TILES = 64;
constexpr float GM_TAIL_BOUNDARY = 0.08f;
static float plain_cost(int M, int N, bool need_sumsq, int align_n) {
    float best = 1e30f;
    for (int i = 0; i < T128x32; ++i) {
        const TileShape& t = kTiles[i];
        if (need_sumsq && !t.sumsq) continue;
        if (align_n % t.bn != 0) continue;
        best = std::min(best, tile_cost(t, M, N));
    }
    return best;
}
static int main_columns(TileId& id, int M, int N, int K, bool need_sumsq, int align_n, float* cost_out = nullptr) {
    if (id == T128x32) return N;
    float best = tile_cost(kTiles[id], M, N);
    int best_n = N;
    struct Report {              // the cost of the plan that is returned
        float* out;
        const float& v;
        ~Report() { if (out) *out = v; }
    } report{cost_out, best};
    for (int i = 0; i < T128x32; ++i) {
        const TileShape& t = kTiles[i];
        if (need_sumsq && !t.sumsq) continue;
        if (align_n % t.bn != 0) continue;
        const int tiles_m = (M + t.bm - 1) / t.bm, tiles_n = (N + t.bn - 1) / t.bn;
        const int rounds = (tiles_m * tiles_n + 255) / 256;
        if (rounds < 2) continue;
        const int keep_n = (rounds - 1) * 256 / tiles_m;              // column tiles that fill the whole rounds
        if (keep_n < 1 || keep_n >= tiles_n) continue;
        const bool small_tail = (tiles_n - keep_n) * tiles_m <= GM_TAIL_MAX_TILES;
        // (a large tail is priced as a plain launch: with at most 1024 rows it would be cut into k-slices instead;
        // and the tail of a pair must start where the second matrix does, or stay inside it: it is one launch)
        if (!small_tail && (M <= 1024 || (align_n != 768 && keep_n * t.bn < align_n))) continue;
        const float tail = small_tail ? 0.3f
                                      : plain_cost(M, N - keep_n * t.bn, need_sumsq, 768) + GM_TAIL_BOUNDARY;
        const float c = (float)(rounds - 1) * (float)(t.bm * t.bn) / (65536.0f * t.rate) + tail;
        if (c < best) {
            best = c;
            best_n = keep_n * t.bn;
            id = (TileId)i;
        }
    }
    return best_n;
}

static int launch_tile(TileId id, const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y,
                       int64_t y_stride, const uint16_t* res, int64_t res_stride, int M, int N, int K,
                       float* sumsq_parts, const uint16_t* w2, uint16_t* y2, int n_split, hipStream_t s) {
#define VITCOP_TILE(BM, BN, WM, WN) \
    return launch_gemm_k<BM, BN, WM, WN, GM_EPI_BF16>(K, x, x_stride, w, y, y_stride, res, res_stride, M, N, K, \
                                                      sumsq_parts, w2, y2, n_split, s)
    switch (id) {
        case T256x256: VITCOP_TILE(256, 256, 2, 2);
        case T192x256: VITCOP_TILE(192, 256, 2, 2);
        case T256x128: VITCOP_TILE(256, 128, 2, 2);
        case T192x128: VITCOP_TILE(192, 128, 2, 2);
        case T128x128: VITCOP_TILE(128, 128, 2, 2);
        case T128x128R: VITCOP_TILE(128, 128, 4, 1);
        default:
            return launch_gemm_cfg<128, 32, 4, 1, 64>(x, x_stride, w, y, y_stride, res, res_stride, M, N, K, sumsq_parts,
                                                      w2, y2, n_split, s);
    }
#undef VITCOP_TILE
}

int launch_gemm(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y,
                int64_t y_stride, const uint16_t* res, int64_t res_stride, int M, int N,
                int K, float* sumsq_parts, hipStream_t s) {
    if (M == 0 || N == 0) return VITCOP_OK;
    const TileId id = choose_tile(M, N, K, sumsq_parts != nullptr, 768 /* any tile width divides it */);
    return launch_tile(id, x, x_stride, w, y, y_stride, res, res_stride, M, N, K, sumsq_parts, nullptr,
                       nullptr, 0, s);
}

// Two projections of the same input in one launch: y1 = x W1^T [M,N1], y2 = x W2^T [M,N2].
// Both outputs are dense and the kernel takes one output row stride, so the fused launch needs
// N1 == N2, and N1 a multiple of the tile width so that no tile straddles the two outputs;
// otherwise two launches.
int launch_gemm_pair(const uint16_t* x, int64_t x_stride, const uint16_t* w1, uint16_t* y1, int N1,
                     const uint16_t* w2, uint16_t* y2, int N2, int M, int K, hipStream_t s) {
    if (M == 0) return VITCOP_OK;
    if (N1 != N2 || N1 % 128 != 0) {
        int rc = launch_gemm(x, x_stride, w1, y1, N1, nullptr, 0, M, N1, K, nullptr, s);
        if (rc) return rc;
        return launch_gemm(x, x_stride, w2, y2, N2, nullptr, 0, M, N2, K, nullptr, s);
    }
    const TileId id = choose_tile(M, N1 + N2, K, false, N1);
    return launch_tile(id, x, x_stride, w1, y1, N1, nullptr, 0, M, N1 + N2, K, nullptr, w2, y2, N1, s);
}

// Split-K for a few hundred to a thousand rows: there are then too few large tiles to fill the chip,
// and 128 x 128 tiles, which would, load twice the bytes per FLOP through a CU's load path, which is
// what bounds them.  So the tiles stay 192 or 256 rows tall and the k-range is cut into `splits` slices
// (blockIdx.y) whose fp32 partials the few-row path's reduction kernels add up.
struct SplitKPlan {
    int bm = 0, bn = 256, splits = 0;          // splits == 0: does not apply
};
static SplitKPlan splitk_plan(int M, int N, int K) {
    SplitKPlan p;
    if (M <= 256 || M > 1024 || N % 16 != 0 || K % 32 != 0) return p;
    // 128-column tiles first: for the same number of workgroups they need half the slices of the 256-column
    // tiles, i.e. half the fp32 partials to write and to add up, and at these sizes that traffic, not the
    // matrix cores, sets the time (317 x 4096 x 4096: 28 us with 2 x 32 tiles x 4 slices against 36 us with
    // 2 x 16 tiles x 8).  Rows per tile: 192 or 256, whichever leaves the shorter slice per workgroup at its
    // measured rate.
    const int t256 = (M + 255) / 256, t192 = (M + 191) / 192, cols = (N + 127) / 128;
    auto slices = [&](int tiles) { return std::min(std::min(16, 256 / std::max(tiles, 1)), K / 32 / 8); };
    const int s192 = slices(t192 * cols), s256 = slices(t256 * cols);
    const float c192 = s192 >= 2 ? 192.0f / (0.89f * (float)s192) : 1e30f;
    const float c256 = s256 >= 2 ? 256.0f / (0.88f * (float)s256) : 1e30f;
    const int s128 = c192 <= c256 ? s192 : s256;
    // (not with slices longer than 4096 of k: inside a layer the 640-row down projection, K = 11008, takes
    // 110 us as 4 x 32 tiles x 2 slices against 91 us as 3 x 16 tiles x 5)
    if (s128 >= 2 && K / s128 <= 4096) {
        p.bn = 128;
        p.bm = c192 <= c256 ? 192 : 256;
        p.splits = s128;
        return p;
    }
    // 256-column tiles: 256 or 192 rows, whichever pads M less (192 runs at 0.9 of the rate)
    const int bm = (float)(t192 * 192) / 0.9f < (float)(t256 * 256) ? 192 : 256;
    const int tiles = (bm == 192 ? t192 : t256) * ((N + 255) / 256);
    const int splits = slices(tiles);                                       // at least 8 k-steps per slice
    if (splits < 3) return p;
    p.bm = bm;
    p.splits = splits;
    return p;
}
static size_t splitk_workspace_bytes(int M, int N, int K) {
    const SplitKPlan p = splitk_plan(M, N, K);
    return p.splits ? up256((size_t)p.splits * M * N * 4) : 0;
}

// scratch of the trailing columns when main_columns cuts the launch (as one matrix, or as the pair N/2 + N/2)
static size_t tail_workspace_bytes(int M, int N, int K) {
    size_t need = 0;
    for (int pair = 0; pair < 2; ++pair) {
        if (pair && N % 256 != 0) break;
        for (int sumsq = 0; sumsq < (pair ? 1 : 2); ++sumsq) {
            TileId id = choose_tile(M, N, K, sumsq != 0, pair ? N / 2 : 768);
            const int n_main = main_columns(id, M, N, K, sumsq != 0, pair ? N / 2 : 768);
            if (n_main < N)
                need = std::max(need, std::max(gemm_skinny_workspace_bytes(M, N - n_main, K),
                                               splitk_workspace_bytes(M, N - n_main, K)));
        }
    }
    return need;
}

size_t gemm_workspace_bytes(int M, int N, int K) {
    const size_t whole = std::max(gemm_skinny_workspace_bytes(M, N, K), splitk_workspace_bytes(M, N, K));
    return whole ? whole : tail_workspace_bytes(M, N, K);
}

// y = x W^T (+ res) by split-K (splitk_plan applies, ws holds splitk_workspace_bytes); optionally the
// norm side output or the RMSNorm of the finished rows, as in the few-row path.
static int launch_gemm_splitk(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y, int64_t y_stride,
                              const uint16_t* res, int64_t res_stride, int M, int N, int K, float* sumsq_parts,
                              void* ws, hipStream_t s, const uint16_t* ln_w, float eps, uint16_t* norm_out,
                              int64_t norm_stride, const uint16_t* w2 = nullptr, uint16_t* y2 = nullptr,
                              int n_split = 0, SkParts* parts_out = nullptr) {
    const SplitKPlan p = splitk_plan(M, N, K);
    float* part = static_cast<float*>(ws);
    int rc;
#define VITCOP_SPLITK(BM, BN)                                                                                    \
    rc = launch_gemm_k<BM, BN, 2, 2, GM_EPI_PART>(K, x, x_stride, w, nullptr, 0, nullptr, 0, M, N, K, nullptr, w2,   \
                                                  nullptr, n_split, s, K, nullptr, nullptr, part, N, p.splits, 0, 0, \
                                                  (int64_t)M * N)
    if (p.bm == 256 && p.bn == 256) VITCOP_SPLITK(256, 256);
    else if (p.bm == 192 && p.bn == 256) VITCOP_SPLITK(192, 256);
    else if (p.bm == 256) VITCOP_SPLITK(256, 128);
    else VITCOP_SPLITK(192, 128);
#undef VITCOP_SPLITK
    if (rc) return rc;
    const SkParts parts{part, 0, p.splits, N, M};
    if (parts_out) {                             // the caller finishes the rows itself
        *parts_out = parts;
        return VITCOP_OK;
    }
    const SkMats mats{{w, w2 ? w2 : w, w}, {y, w2 ? y2 : y, y}, {y_stride, y_stride, y_stride},
                      {w2 ? n_split : N, N, N}};
    return launch_partial_reduce(parts, N, mats, res, res_stride, sumsq_parts, ln_w, eps, norm_out, norm_stride,
                                 nullptr, s);
}

int launch_gemm_ws(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y, int64_t y_stride,
                   const uint16_t* res, int64_t res_stride, int M, int N, int K, float* sumsq_parts, void* ws,
                   size_t ws_bytes, hipStream_t s) {
    if (M == 0 || N == 0) return VITCOP_OK;
    // one to four rows: a stream over W with no partial sums to reduce
    if (!sumsq_parts && gemv_applies(M, K) && N % 2 == 0 && x_stride % 8 == 0 && y_stride % 2 == 0 &&
        (!res || res_stride % 2 == 0))
        return launch_gemv(x, x_stride, nullptr, 0.f, w, y, y_stride, res, res_stride, M, N, K, s);
    const size_t need = gemm_skinny_workspace_bytes(M, N, K);
    if (ws && need && ws_bytes >= need)
        return launch_gemm_skinny(x, x_stride, w, y, y_stride, res, res_stride, M, N, K, sumsq_parts, nullptr,
                                  nullptr, 0, ws, s);
    const size_t need_k = splitk_workspace_bytes(M, N, K);
    if (ws && need_k && ws_bytes >= need_k)
        return launch_gemm_splitk(x, x_stride, w, y, y_stride, res, res_stride, M, N, K, sumsq_parts, ws, s, nullptr,
                                  0.f, nullptr, 0);
    if (ws) {               // a few tiles over whole rounds: leading columns on the big tiles, the rest on their own
        TileId id = choose_tile(M, N, K, sumsq_parts != nullptr, 768);
        const int n_main = main_columns(id, M, N, K, sumsq_parts != nullptr, 768);
        const size_t need_tail = n_main < N ? std::max(gemm_skinny_workspace_bytes(M, N - n_main, K),
                                                       splitk_workspace_bytes(M, N - n_main, K))
                                            : 0;
        if (n_main < N && ws_bytes >= need_tail) {
            int rc = launch_tile(id, x, x_stride, w, y, y_stride, res, res_stride, M, n_main, K, sumsq_parts, nullptr,
                                 nullptr, 0, s);
            if (rc) return rc;
            return launch_gemm_ws(x, x_stride, w + (int64_t)n_main * K, y + n_main, y_stride,
                                  res ? res + n_main : nullptr, res_stride, M, N - n_main, K,
                                  sumsq_parts ? sumsq_parts + (int64_t)(n_main / GM_PART) * M : nullptr, ws, ws_bytes, s);
        }
    }
    return launch_gemm(x, x_stride, w, y, y_stride, res, res_stride, M, N, K, sumsq_parts, s);
}

int launch_gemm_norm_ws(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y, int64_t y_stride,
                        const uint16_t* res, int64_t res_stride, int M, int N, int K, const uint16_t* ln_w,
                        float eps, uint16_t* norm_out, int64_t norm_stride, void* ws, size_t ws_bytes,
                        hipStream_t s) {
    if (M == 0 || N == 0) return VITCOP_OK;
    const size_t need = gemm_skinny_workspace_bytes(M, N, K);
    if (ws && need && ws_bytes >= need && gemm_skinny_fuses_norm(M, N, K))
        return launch_gemm_skinny(x, x_stride, w, y, y_stride, res, res_stride, M, N, K, nullptr, nullptr, nullptr, 0,
                                  ws, s, ln_w, eps, norm_out, norm_stride);
    const size_t need_k = splitk_workspace_bytes(M, N, K);
    if (ws && need_k && ws_bytes >= need_k && partial_reduce_fuses_norm(N))
        return launch_gemm_splitk(x, x_stride, w, y, y_stride, res, res_stride, M, N, K, nullptr, ws, s, ln_w, eps,
                                  norm_out, norm_stride);
    int rc = launch_gemm_ws(x, x_stride, w, y, y_stride, res, res_stride, M, N, K, nullptr, ws, ws_bytes, s);
    if (rc) return rc;
    return launch_rmsnorm(y, y_stride, ln_w, eps, norm_out, norm_stride, M, N, s);
}

// out = silu(x Wg^T) * (x Wu^T) as ONE launch of the big tiles: a tile's columns are half gate, half up, and the
// epilogue applies the activation (GM_EPI_GATED), so gate and up never reach memory.
// (F columns of an output whose rows are out_stride apart)
static int launch_tile_gated(TileId id, const uint16_t* x, int64_t x_stride, const uint16_t* wg, const uint16_t* wu,
                             uint16_t* out, int64_t out_stride, int M, int F, int K, hipStream_t s) {
#define VITCOP_GATED(BM, BN) \
    return launch_gemm_k<BM, BN, 2, 2, GM_EPI_GATED>(K, x, x_stride, wg, out, out_stride, nullptr, 0, M, F, K, nullptr, \
                                                     wu, nullptr, 0, s)
    switch (id) {
        case T256x256: VITCOP_GATED(256, 256);
        case T192x256: VITCOP_GATED(192, 256);
        case T256x128: VITCOP_GATED(256, 128);
        case T192x128: VITCOP_GATED(192, 128);
        case T192x192G: VITCOP_GATED(192, 192);
        default: VITCOP_GATED(128, 128);
    }
#undef VITCOP_GATED
}

int launch_gemm_gated_ws(const uint16_t* x, int64_t x_stride, const uint16_t* wg, const uint16_t* wu, int F,
                         uint16_t* gate, uint16_t* up, uint16_t* out, int M, int K, void* ws, size_t ws_bytes,
                         hipStream_t s) {
    if (M == 0 || F == 0) return VITCOP_OK;
    const size_t need = gemm_skinny_workspace_bytes(M, 2 * F, K);
    if (ws && need && ws_bytes >= need && F % 128 == 0)
        return launch_gemm_skinny_gated(x, x_stride, wg, wu, F, out, M, K, ws, s);
    // more rows than the few-row kernel takes: the big tiles with the activation in their epilogue, unless the
    // launch is one that gets cut into k-slices or sends a few trailing tiles down a path of their own (a few
    // hundred rows): those produce gate and up separately.  A large tail (many rows, whole rounds plus a part
    // of one) stays on this path: first the columns that fill the whole rounds, then the rest on the tiles
    // that suit it.
    if (F % 8 == 0 && splitk_plan(M, 2 * F, K).splits == 0) {
        const uint16_t *g_w = wg, *u_w = wu;
        uint16_t* o = out;
        int f_left = F;
        bool fused = true;
        while (f_left > 0) {
            TileId id = choose_tile(M, 2 * f_left, K, false, 768);
            if (id == T128x128R) id = T128x128;
            const bool first = f_left == F;              // only the whole launch may still go the separate way
            if (!(id == T256x256 || id == T192x256 || id == T256x128 || id == T192x128 || id == T128x128)) {
                if (first) {
                    fused = false;
                    break;
                }
                id = T128x128;
            }
            TileId cut_id = id;
            float cut_cost = 0.f;
            int n_main = ws && f_left % 128 == 0 ? main_columns(cut_id, M, 2 * f_left, K, false, 768, &cut_cost)
                                                 : 2 * f_left;
            // (the 192 x 192 tiles exist in this form only: a cut must beat them too)
            if (cut_id == T128x128R || cut_cost >= tile_cost(kTiles[T192x192G], M, 2 * f_left)) n_main = 2 * f_left;
            int f_now = f_left;
            if (n_main < 2 * f_left) {
                const TileShape& t = kTiles[cut_id];
                const int tail_tiles = (2 * f_left - n_main + t.bn - 1) / t.bn * ((M + t.bm - 1) / t.bm);
                if (tail_tiles <= GM_TAIL_MAX_TILES && first) {  // the small-tail cut: separate gate and up
                    fused = false;
                    break;
                }
                if (tail_tiles > GM_TAIL_MAX_TILES) {
                    id = cut_id;
                    f_now = n_main / 2;
                }
            } else if (tile_cost(kTiles[T192x192G], M, 2 * f_left) < tile_cost(kTiles[id], M, 2 * f_left)) {
                // a few hundred rows leave the 256-column tiles a third of the CUs short (317 x 22016: 172
                // tiles); 192 x 192 tiles (230) fill them
                id = T192x192G;
            }
            int rc = launch_tile_gated(id, x, x_stride, g_w, u_w, o, F, M, f_now, K, s);
            if (rc) return rc;
            g_w += (int64_t)f_now * K;
            u_w += (int64_t)f_now * K;
            o += f_now;
            f_left -= f_now;
        }
        if (fused) return VITCOP_OK;
    }
    int rc = launch_gemm_pair_ws(x, x_stride, wg, gate, F, wu, up, F, M, K, ws, ws_bytes, s);
    if (rc) return rc;
    return launch_silu_mul(gate, up, out, (int64_t)M * F, s);
}

int launch_gemm_triple_ws(const uint16_t* x, int64_t x_stride, const uint16_t* const w[3], uint16_t* const y[3],
                          const int n[3], int M, int K, void* ws, size_t ws_bytes, hipStream_t s) {
    if (M == 0) return VITCOP_OK;
    const size_t need = gemm_skinny_workspace_bytes(M, n[0] + n[1] + n[2], K);
    if (ws && need && ws_bytes >= need && n[0] % 128 == 0 && n[1] % 128 == 0)
        return launch_gemm_skinny3(x, x_stride, w, y, n, M, K, ws, s);
    int rc = launch_gemm_ws(x, x_stride, w[0], y[0], n[0], nullptr, 0, M, n[0], K, nullptr, ws, ws_bytes, s);
    if (rc) return rc;
    return launch_gemm_pair_ws(x, x_stride, w[1], y[1], n[1], w[2], y[2], n[2], M, K, ws, ws_bytes, s);
}

int launch_gemm_pair_ws(const uint16_t* x, int64_t x_stride, const uint16_t* w1, uint16_t* y1, int N1,
                        const uint16_t* w2, uint16_t* y2, int N2, int M, int K, void* ws, size_t ws_bytes,
                        hipStream_t s) {
    if (M == 0) return VITCOP_OK;
    const size_t need = gemm_skinny_workspace_bytes(M, N1 + N2, K);
    if (ws && need && ws_bytes >= need && N1 == N2 && N1 % 128 == 0)
        return launch_gemm_skinny(x, x_stride, w1, y1, N1, nullptr, 0, M, N1 + N2, K, nullptr, w2, y2, N1, ws, s);
    const size_t need_k = splitk_workspace_bytes(M, N1 + N2, K);
    if (ws && need_k && ws_bytes >= need_k && N1 == N2 && N1 % 256 == 0)      // no tile straddles the two outputs
        return launch_gemm_splitk(x, x_stride, w1, y1, N1, nullptr, 0, M, N1 + N2, K, nullptr, ws, s, nullptr, 0.f,
                                  nullptr, 0, w2, y2, N1);
    if (ws && N1 == N2 && N1 % 128 == 0) {       // the same cut for the pair: the tail lies in the second matrix
        const int N = N1 + N2;
        TileId id = choose_tile(M, N, K, false, N1);
        const int n_main = main_columns(id, M, N, K, false, N1);
        const bool cut = n_main < N && n_main >= N1;
        const size_t need_tail = cut ? std::max(gemm_skinny_workspace_bytes(M, N - n_main, K),
                                                splitk_workspace_bytes(M, N - n_main, K))
                                     : 0;
        if (cut && ws_bytes >= need_tail) {
            int rc = launch_tile(id, x, x_stride, w1, y1, N1, nullptr, 0, M, n_main, K, nullptr, w2, y2, N1, s);
            if (rc) return rc;
            return launch_gemm_ws(x, x_stride, w2 + (int64_t)(n_main - N1) * K, y2 + (n_main - N1), N2, nullptr, 0, M,
                                  N - n_main, K, nullptr, ws, ws_bytes, s);
        }
    }
    return launch_gemm_pair(x, x_stride, w1, y1, N1, w2, y2, N2, M, K, s);
}

// Which way launch_gemm_qkv_rope_ws goes at M rows: 1 the three matrices in one few-row launch, 2 split-K of K
// and of the Q/V pair with their partial sums side by side in ws, 0 the plain sequence.
static int qkv_path(int M, int qd, int kd, int d, int K) {
    if (d != 64 && d != 128) return 0;
    if (gemm_skinny_workspace_bytes(M, kd + qd + kd, K) && kd % 128 == 0 && qd % 128 == 0) return 1;
    if (splitk_workspace_bytes(M, kd, K) && splitk_workspace_bytes(M, qd + kd, K) && qd == kd && kd % 256 == 0)
        return 2;
    return 0;
}

size_t gemm_qkv_workspace_bytes(int M, int Hq, int Hkv, int d, int K) {
    const int qd = Hq * d, kd = Hkv * d;
    size_t need = std::max(gemm_workspace_bytes(M, kd, K), gemm_workspace_bytes(M, qd + kd, K));
    need = std::max(need, gemm_workspace_bytes(M, kd + qd + kd, K));
    if (qkv_path(M, qd, kd, d, K) == 2)
        need = std::max(need, splitk_workspace_bytes(M, kd, K) + splitk_workspace_bytes(M, qd + kd, K));
    return need;
}

int launch_gemm_qkv_rope_ws(const uint16_t* x, int64_t x_stride, const uint16_t* wk, const uint16_t* wq,
                            const uint16_t* wv, uint16_t* k, uint16_t* q, uint16_t* v, int Hq, int Hkv, int d,
                            const int32_t* positions, float theta, int M, int K, void* ws, size_t ws_bytes,
                            hipStream_t s) {
    if (M == 0) return VITCOP_OK;
    const int qd = Hq * d, kd = Hkv * d;
    const uint16_t* const w3[3] = {wk, wq, wv};
    uint16_t* const y3[3] = {k, q, v};
    const int n3[3] = {kd, qd, kd};
    const int path = ws ? qkv_path(M, qd, kd, d, K) : 0;
    if (path == 1 && ws_bytes >= gemm_skinny_workspace_bytes(M, kd + qd + kd, K)) {
        SkParts parts{};
        int rc = launch_gemm_skinny3(x, x_stride, w3, y3, n3, M, K, ws, s, &parts);
        if (rc) return rc;
        if (parts.part == nullptr) return launch_rope(q, k, positions, M, Hq, Hkv, d, theta, s);   // written directly
        const QkvParts P{{parts, parts, parts}, {0, kd, kd + qd}};
        return launch_qkv_finish(P, k, q, v, Hq, Hkv, d, positions, theta, s);
    }
    const size_t need_k = splitk_workspace_bytes(M, kd, K), need_qv = splitk_workspace_bytes(M, qd + kd, K);
    if (path == 2 && ws_bytes >= need_k + need_qv) {
        SkParts pk{}, pqv{};
        int rc = launch_gemm_splitk(x, x_stride, wk, k, kd, nullptr, 0, M, kd, K, nullptr, ws, s, nullptr, 0.f, nullptr,
                                    0, nullptr, nullptr, 0, &pk);
        if (rc) return rc;
        rc = launch_gemm_splitk(x, x_stride, wq, q, qd, nullptr, 0, M, qd + kd, K, nullptr,
                                static_cast<char*>(ws) + need_k, s, nullptr, 0.f, nullptr, 0, wv, v, qd, &pqv);
        if (rc) return rc;
        const QkvParts P{{pk, pqv, pqv}, {0, 0, qd}};
        return launch_qkv_finish(P, k, q, v, Hq, Hkv, d, positions, theta, s);
    }
    const int rc = launch_gemm_triple_ws(x, x_stride, w3, y3, n3, M, K, ws, ws_bytes, s);
    if (rc) return rc;
    return launch_rope(q, k, positions, M, Hq, Hkv, d, theta, s);
}

// dist[b][i,j] = ||f_i - f_j||_2 in fp32 between the rows of each of `batch` bf16 matrices
// f [n,K] (row stride and batch stride in elements), with their squared row norms sq given.
// sq must be readable, and the rows of dist writable, up to the next multiple of 4 entries
// (dist_stride % 4 == 0; the pad holds garbage).
int launch_pairwise_dist(const uint16_t* f, int64_t row_stride, int64_t batch_stride, const float* sq,
                         int64_t sq_batch, float* dist, int64_t dist_stride, int64_t dist_batch, int n, int K,
                         int batch, hipStream_t s) {
    if (n == 0 || batch == 0) return VITCOP_OK;
    return launch_gemm_k<128, 128, 2, 2, GM_EPI_DIST>(K, f, row_stride, f, nullptr, 0, nullptr, 0, n, n, K, nullptr,
                                                      nullptr, nullptr, 0, s, row_stride, sq, sq, dist, dist_stride, batch,
                                                      batch_stride, sq_batch, dist_batch);
}

}  // namespace vitcop
