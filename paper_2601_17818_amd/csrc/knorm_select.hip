// K-vector L2-norm saliency (Sec. 3.2.2, Eq. 4) and the Stage III selection
// (Alg. 1: TopK of -K_norms).
//
// knorm_kernel   : HBM-bound stream.  One wavefront reduces one token row
//                  (or several short rows at once) with 16-byte loads, eight
//                  loads in flight per lane, fp32 accumulation.
// select_kernel  : one workgroup per sample; candidates live in LDS as
//                  order-preserving 32-bit keys; radix selection + ordered
//                  emission (select_device.h).
#include "vitcop_internal.h"
#include "device_utils.h"
#include "select_device.h"

namespace vitcop {

constexpr int KN_THREADS = 256;
constexpr int KN_WAVES = KN_THREADS / 64;

// CPL: 16-byte chunks per lane per row (row = 64*CPL chunks = 512*CPL elements).
// G  : rows a wavefront reduces together, so that CPL*G loads are in flight.
template <int CPL, int G>
__global__ __launch_bounds__(KN_THREADS) void knorm_kernel(
    const uint16_t* __restrict__ k, int64_t row_stride, int64_t batch_stride, int vis_start,
    int n_vis, float* __restrict__ norms) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int row0 = (blockIdx.x * KN_WAVES + wv) * G;
    if (row0 >= n_vis) return;
    const uint16_t* base = k + (int64_t)b * batch_stride + (int64_t)(vis_start + row0) * row_stride;
    uint4 v[G][CPL];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        // rows past the end re-read the last row; their result is not stored
        const int r = min(row0 + g, n_vis - 1) - row0;
        const uint4* p = reinterpret_cast<const uint4*>(base + (int64_t)r * row_stride) + lane;
#pragma unroll
        for (int c = 0; c < CPL; ++c) v[g][c] = ld_nt16(p + 64 * c);
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int c = 0; c < CPL; c += 2) {
            a0 = sumsq8(v[g][c], a0);
            if (c + 1 < CPL) a1 = sumsq8(v[g][c + 1], a1);
        }
        float s = wave_sum(a0 + a1);
        if (lane == 0 && row0 + g < n_vis) norms[(int64_t)b * n_vis + row0 + g] = sqrtf(s);
    }
}

// Any row length that is a multiple of 8 elements: one wavefront per row.
__global__ __launch_bounds__(KN_THREADS) void knorm_generic_kernel(
    const uint16_t* __restrict__ k, int64_t row_stride, int64_t batch_stride, int chunks,
    int vis_start, int n_vis, float* __restrict__ norms) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int row = blockIdx.x * KN_WAVES + wv;
    if (row >= n_vis) return;
    const uint4* p = reinterpret_cast<const uint4*>(k + (int64_t)b * batch_stride +
                                                    (int64_t)(vis_start + row) * row_stride);
    float a = 0.f;
    for (int c = lane; c < chunks; c += 64) a = sumsq8(p[c], a);
    a = wave_sum(a);
    if (lane == 0) norms[(int64_t)b * n_vis + row] = sqrtf(a);
}

__global__ __launch_bounds__(SEL_THREADS) void select_smallest_kernel(
    const float* __restrict__ parts, int n_parts, int64_t part_stride, int64_t sample_stride,
    int64_t offset, int do_sqrt, float* __restrict__ norms_out, int T, int vis_start, int n_vis_max,
    int keep_max, int32_t* __restrict__ keep_idx, const int32_t* __restrict__ n_vis_samples,
    int32_t* __restrict__ n_vis_samples_out) {
    extern __shared__ unsigned sel_keys[];
    __shared__ SelectShared sh;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int Tp = T - n_vis_max + keep_max;
    int32_t* out = keep_idx + (int64_t)b * Tp;
    // A right-padded batch: this sample has n_vis of the n_vis_max visual tokens, its text follows them
    // directly, and the last n_vis_max - n_vis rows of its T are padding.  It keeps min(keep_max, n_vis).
    const int n_vis = n_vis_samples ? min(max(n_vis_samples[b], 0), n_vis_max) : n_vis_max;
    const int keep = min(keep_max, n_vis);
    const int T_real = T - (n_vis_max - n_vis);
    const float* src = parts + (int64_t)b * sample_stride + offset;
    // Four candidates per thread at a time, eight parts each: 32 independent loads in flight per round trip
    // (the workgroup is alone on its CU and the reads are all latency); every candidate's parts are added in
    // index order, so the sums do not depend on the grouping.
    constexpr int RU = 4;
    for (int i0 = tid; i0 < n_vis; i0 += SEL_THREADS * RU) {
        int row[RU];
        float v[RU];
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            row[r] = min(i0 + r * SEL_THREADS, n_vis - 1);      // past the end: a valid row, not stored
            v[r] = 0.f;                                         // (0 + part 0 is part 0 exactly)
        }
        for (int p = 0; p < n_parts; p += 8) {                  // the last group may be short: its loads repeat
            float w[RU][8];                                     // the last part and are not added
#pragma unroll
            for (int r = 0; r < RU; ++r)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    w[r][j] = src[(int64_t)min(p + j, n_parts - 1) * part_stride + row[r]];
#pragma unroll
            for (int r = 0; r < RU; ++r)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (p + j < n_parts) v[r] += w[r][j];
        }
#pragma unroll
        for (int r = 0; r < RU; ++r) {
            const int i = i0 + r * SEL_THREADS;
            if (i >= n_vis) continue;
            const float val = do_sqrt ? sqrtf(v[r]) : v[r];
            if (norms_out) norms_out[(int64_t)b * n_vis_max + i] = val;
            sel_keys[i] = __float_as_uint(val);      // val >= 0: bit order = value order
        }
    }
    if (norms_out)
        for (int i = n_vis + tid; i < n_vis_max; i += SEL_THREADS) norms_out[(int64_t)b * n_vis_max + i] = 0.f;
    // text before and after the visual span is always kept; padding rows of the output name the last row
    for (int i = tid; i < vis_start; i += SEL_THREADS) out[i] = i;
    for (int i = vis_start + n_vis + tid; i < T_real; i += SEL_THREADS) out[i - n_vis + keep] = i;
    for (int j = T_real - n_vis + keep + tid; j < Tp; j += SEL_THREADS) out[j] = T - 1;
    if (n_vis_samples_out && tid == 0) n_vis_samples_out[b] = keep;
    __syncthreads();
    block_select_emit(sel_keys, n_vis, keep, out + vis_start, vis_start, sh);
}

int launch_knorm(const uint16_t* k, int64_t row_stride, int64_t batch_stride, int B,
                 int row_elems, int vis_start, int n_vis, float* norms, hipStream_t s) {
    if (B == 0 || n_vis == 0) return VITCOP_OK;
    const int chunks = row_elems / 8;
#define VITCOP_KN(CPL, G)                                                                     \
    do {                                                                                      \
        dim3 grid((n_vis + KN_WAVES * (G) - 1) / (KN_WAVES * (G)), B);                        \
        hipLaunchKernelGGL((knorm_kernel<CPL, G>), grid, dim3(KN_THREADS), 0, s, k,           \
                           row_stride, batch_stride, vis_start, n_vis, norms);                \
    } while (0)
    switch (chunks) {
        case 64:  VITCOP_KN(1, 8); break;    //  512 elements (GQA 4 x 128)
        case 128: VITCOP_KN(2, 4); break;    // 1024
        case 256: VITCOP_KN(4, 2); break;    // 2048
        case 512: VITCOP_KN(8, 1); break;    // 4096 (MHA 32 x 128)
        case 1024: VITCOP_KN(16, 1); break;  // 8192
        default: {
            dim3 grid((n_vis + KN_WAVES - 1) / KN_WAVES, B);
            hipLaunchKernelGGL(knorm_generic_kernel, grid, dim3(KN_THREADS), 0, s, k, row_stride,
                               batch_stride, chunks, vis_start, n_vis, norms);
        }
    }
#undef VITCOP_KN
    return launch_status("knorm");
}

int launch_select_smallest(const float* parts, int n_parts, int64_t part_stride,
                           int64_t sample_stride, int64_t offset, int do_sqrt,
                           float* norms_out, int B, int T, int vis_start, int n_vis,
                           int keep, int32_t* keep_idx, hipStream_t s, const int32_t* n_vis_samples,
                           int32_t* n_vis_samples_out) {
    if (B == 0 || T - n_vis + keep == 0) return VITCOP_OK;
    const size_t smem = (size_t)(n_vis > 0 ? n_vis : 1) * sizeof(unsigned);
    if (smem > 48 * 1024) {
        int rc = hip_status(hipFuncSetAttribute((const void*)select_smallest_kernel,
                                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                                (int)smem),
                            "hipFuncSetAttribute(select)");
        if (rc) return rc;
    }
    hipLaunchKernelGGL(select_smallest_kernel, dim3(B), dim3(SEL_THREADS), smem, s, parts,
                       n_parts, part_stride, sample_stride, offset, do_sqrt, norms_out, T,
                       vis_start, n_vis, keep, keep_idx, n_vis_samples, n_vis_samples_out);
    return launch_status("select_smallest");
}

}  // namespace vitcop
