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
#include "vitcop_internal.h"
#include "device_utils.h"

namespace vitcop {

constexpr int GM_THREADS = 256;
constexpr int GM_BK = 32;
constexpr int GM_LD = GM_BK + 8;     // bf16 per LDS row (80 B: conflict-free 16 B reads)
constexpr int GM_PART = 128;         // columns per sum-of-squares partial

template <int BM, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(GM_THREADS) void gemm_kernel(
    const uint16_t* __restrict__ x, int64_t x_stride, const uint16_t* __restrict__ w,
    uint16_t* __restrict__ y, int64_t y_stride, const uint16_t* __restrict__ res,
    int64_t res_stride, int M, int N, int K, float* __restrict__ sumsq_parts) {
    static_assert(WAVES_M * WAVES_N == 4, "four wavefronts");
    constexpr int TM = BM / WAVES_M, TN = BN / WAVES_N;
    constexpr int MI = TM / 32, NI = TN / 32;
    static_assert(TN == GM_PART, "one sum-of-squares partial per wavefront");
    constexpr int XCH = BM * GM_BK / 8 / GM_THREADS;   // 16-byte chunks per thread
    constexpr int WCH = BN * GM_BK / 8 / GM_THREADS;

    __shared__ __attribute__((aligned(16))) uint16_t Xs[BM * GM_LD];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[BN * GM_LD];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int wm = wv % WAVES_M, wn = wv / WAVES_M;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    f32x16 acc[NI][MI];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < MI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    u32x4 xr[XCH], wr[WCH];
    auto load_tile = [&](int k0) {
#pragma unroll
        for (int j = 0; j < XCH; ++j) {
            const int id = tid + GM_THREADS * j;
            const int row = min(m0 + (id >> 2), M - 1);
            xr[j] = *reinterpret_cast<const u32x4*>(x + (int64_t)row * x_stride + k0 + (id & 3) * 8);
        }
#pragma unroll
        for (int j = 0; j < WCH; ++j) {
            const int id = tid + GM_THREADS * j;
            const int row = min(n0 + (id >> 2), N - 1);
            wr[j] = *reinterpret_cast<const u32x4*>(w + (int64_t)row * K + k0 + (id & 3) * 8);
        }
    };
    load_tile(0);

    for (int k0 = 0; k0 < K; k0 += GM_BK) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < XCH; ++j) {
            const int id = tid + GM_THREADS * j;
            *reinterpret_cast<u32x4*>(&Xs[(id >> 2) * GM_LD + (id & 3) * 8]) = xr[j];
        }
#pragma unroll
        for (int j = 0; j < WCH; ++j) {
            const int id = tid + GM_THREADS * j;
            *reinterpret_cast<u32x4*>(&Ws[(id >> 2) * GM_LD + (id & 3) * 8]) = wr[j];
        }
        __syncthreads();
        if (k0 + GM_BK < K) load_tile(k0 + GM_BK);
#pragma unroll
        for (int kc = 0; kc < GM_BK / 16; ++kc) {
            bf16x8 xf[MI], wf[NI];
#pragma unroll
            for (int j = 0; j < MI; ++j)
                xf[j] = *reinterpret_cast<const bf16x8*>(
                    &Xs[(wm * TM + j * 32 + l32) * GM_LD + kc * 16 + g * 8]);
#pragma unroll
            for (int i = 0; i < NI; ++i)
                wf[i] = *reinterpret_cast<const bf16x8*>(
                    &Ws[(wn * TN + i * 32 + l32) * GM_LD + kc * 16 + g * 8]);
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < MI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
        }
    }

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

int launch_gemm(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y,
                int64_t y_stride, const uint16_t* res, int64_t res_stride, int M, int N,
                int K, float* sumsq_parts, hipStream_t s) {
    if (M == 0 || N == 0) return VITCOP_OK;
    // large problems: 256x256 tiles (each wavefront 128x128); otherwise 128x128 tiles
    const long big_tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
    if (big_tiles >= 192) {
        dim3 grid((N + 255) / 256, (M + 255) / 256);
        hipLaunchKernelGGL((gemm_kernel<256, 256, 2, 2>), grid, dim3(GM_THREADS), 0, s, x, x_stride,
                           w, y, y_stride, res, res_stride, M, N, K, sumsq_parts);
    } else {
        dim3 grid((N + 127) / 128, (M + 127) / 128);
        hipLaunchKernelGGL((gemm_kernel<128, 128, 4, 1>), grid, dim3(GM_THREADS), 0, s, x, x_stride,
                           w, y, y_stride, res, res_stride, M, N, K, sumsq_parts);
    }
    return launch_status("gemm");
}

}  // namespace vitcop
