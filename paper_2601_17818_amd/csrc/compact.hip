// Compaction of the surviving tokens: dst[b,j,:] = src[b, idx[b,j], :] for up
// to eight tensors in one launch (the token removal implied by
// TopK(V_current, ...) in Alg. 1).  Pure HBM copy: 16-byte loads and stores,
// one workgroup per (output row, tensor).
#include "vitcop_internal.h"
#include "device_utils.h"

namespace vitcop {

struct GatherArgs {
    vitcop_gather_t t[VITCOP_MAX_GATHER];
};

constexpr int CP_THREADS = 256;

__global__ __launch_bounds__(CP_THREADS) void compact_kernel(GatherArgs a,
                                                            const int32_t* __restrict__ idx,
                                                            int T_out) {
    const vitcop_gather_t g = a.t[blockIdx.y];
    const int64_t row = blockIdx.x;                 // b * T_out + j
    const int b = (int)(row / T_out);
    const int src_row = idx[row];
    const char* src = (const char*)g.src + (int64_t)b * g.src_batch_stride_bytes +
                      (int64_t)src_row * g.src_row_stride_bytes;
    char* dst = (char*)g.dst + row * g.row_bytes;
    const bool vec = ((g.row_bytes | g.src_row_stride_bytes | g.src_batch_stride_bytes |
                       (int64_t)(uintptr_t)g.src | (int64_t)(uintptr_t)g.dst) & 15) == 0;
    if (vec) {
        const int n = (int)(g.row_bytes >> 4);
        const uint4* s4 = (const uint4*)src;
        uint4* d4 = (uint4*)dst;
        for (int i = threadIdx.x; i < n; i += CP_THREADS)
            st_nt16(d4 + i, ld_nt16(s4 + i));
    } else {
        const int n = (int)(g.row_bytes >> 2);
        const uint32_t* s1 = (const uint32_t*)src;
        uint32_t* d1 = (uint32_t*)dst;
        for (int i = threadIdx.x; i < n; i += CP_THREADS) d1[i] = s1[i];
    }
}

int launch_compact(const vitcop_gather_t* t, int n, const int32_t* idx, int B, int T_out,
                   hipStream_t s) {
    if (n == 0 || B == 0 || T_out == 0) return VITCOP_OK;
    GatherArgs a;
    for (int i = 0; i < VITCOP_MAX_GATHER; ++i) a.t[i] = t[i < n ? i : 0];
    dim3 grid((unsigned)((int64_t)B * T_out), n);
    hipLaunchKernelGGL(compact_kernel, grid, dim3(CP_THREADS), 0, s, a, idx, T_out);
    return launch_status("compact");
}

}  // namespace vitcop
