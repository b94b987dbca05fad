// Visual-textual collaborative pruning and merging (Sec. 3.2.3, Eq. 5-6; Alg. 3 of arXiv
// 2601.17818): inside every cluster of visual tokens the q_c tokens with the smallest K-vector
// norm survive as "elites", the rest of the cluster is averaged into one merged token.
//
//   1. collab_rank_kernel   per token: size of its cluster and its rank inside it by
//                           (K-norm, index) ascending -> elite iff rank < q_c, with
//                           q_c = floor(|C_c| (B - N_c) / n)                       (Eq. 5)
//   2. collab_plan_kernel   per image: output row of every token (elites in ascending
//                           token index, then one merged row per cluster that has
//                           non-elites, in cluster order), row count, representative
//                           token of each row
//   3. collab_emit_kernel   per output row: copy of the elite, or the mean of the
//                           absorbed tokens (fp32 sums in ascending token order)   (Eq. 6)
//
// Everything is integer work on the given labels and fp32 norms except the means, so the
// result is deterministic; ties in the norm go to the lower index.
#include <atomic>
#include "vitcop_internal.h"
#include "device_utils.h"

namespace vitcop {

constexpr int CB_ROW_THREADS = 256;      // 4 wavefronts, one token each
constexpr int CB_PLAN_THREADS = 1024;

// B - N_c, not below 0
__device__ __forceinline__ int elite_budget(int budget, int n_clusters) { return max(0, budget - n_clusters); }

__global__ __launch_bounds__(CB_ROW_THREADS) void collab_rank_kernel(
    const int32_t* __restrict__ labels, const float* __restrict__ norms,
    const int32_t* __restrict__ n_clusters, int n, int budget, int32_t* __restrict__ elite) {
    const int b = blockIdx.y, lane = threadIdx.x & 63;
    const int i = blockIdx.x * (CB_ROW_THREADS / 64) + (threadIdx.x >> 6);
    if (i >= n) return;
    labels += (int64_t)b * n;
    norms += (int64_t)b * n;
    const int li = labels[i];
    const float ni = norms[i];
    int size = 0, rank = 0;
    for (int j = lane; j < n; j += 64) {
        const bool same = labels[j] == li;
        const float nj = norms[j];
        size += same ? 1 : 0;
        rank += (same && (nj < ni || (nj == ni && j < i))) ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        size += __shfl_xor(size, o, 64);
        rank += __shfl_xor(rank, o, 64);
    }
    if (lane == 0) {
        const int quota = (int)(((int64_t)size * elite_budget(budget, n_clusters[b])) / n);
        elite[(int64_t)b * n + i] = rank < quota ? 1 : 0;
    }
}

// One workgroup per image.  LDS: has_rest[R] / merged_row[R] and first_rest[R], R <= n.
__global__ __launch_bounds__(CB_PLAN_THREADS) void collab_plan_kernel(
    const int32_t* __restrict__ labels, const int32_t* __restrict__ elite,
    const int32_t* __restrict__ n_clusters, int n, int32_t* __restrict__ assign,
    int32_t* __restrict__ out_index, int32_t* __restrict__ n_out) {
    extern __shared__ __attribute__((aligned(16))) int cb_lds[];
    __shared__ int wave_tot[CB_PLAN_THREADS / 64];
    const int tid = threadIdx.x, b = blockIdx.x;
    labels += (int64_t)b * n;
    elite += (int64_t)b * n;
    assign += (int64_t)b * n;
    out_index += (int64_t)b * n;
    const int R = min(max(n_clusters[b], 0), n);          // labels are the caller's contract; stay inside LDS anyway
    auto label_of = [&](int i) { return min(max(labels[i], 0), max(R - 1, 0)); };
    int* merged_row = cb_lds;            // first: 1 if the cluster has non-elites; then: its output row
    int* first_rest = cb_lds + n;        // lowest token index among the cluster's non-elites
    for (int c = tid; c < R; c += CB_PLAN_THREADS) {
        merged_row[c] = 0;
        first_rest[c] = 0x7fffffff;
    }
    __syncthreads();
    for (int i = tid; i < n; i += CB_PLAN_THREADS)
        if (!elite[i]) {
            merged_row[label_of(i)] = 1;                    // same value from every writer
            atomicMin(&first_rest[label_of(i)], i);
        }
    __syncthreads();

    // elites keep their order: row = number of elites before the token
    const int n_elite = block_exclusive_scan<CB_PLAN_THREADS>(
        0, n, wave_tot, [&](int i) { return elite[i]; },
        [&](int i, int f, int pos) {
            if (f) {
                assign[i] = pos;
                out_index[pos] = i;
            }
        });
    // merged rows follow, one per cluster with non-elites, in cluster order
    const int n_merged = block_exclusive_scan<CB_PLAN_THREADS>(
        0, R, wave_tot, [&](int c) { return merged_row[c]; },
        [&](int c, int f, int pos) {
            if (f) out_index[n_elite + pos] = first_rest[c];
            merged_row[c] = n_elite + pos;
        });
    __syncthreads();
    for (int i = tid; i < n; i += CB_PLAN_THREADS)
        if (!elite[i]) assign[i] = merged_row[label_of(i)];
    if (tid == 0) n_out[b] = n_elite + n_merged;
}

// One workgroup per (output row, image); a thread owns 8 channels.
__global__ __launch_bounds__(256) void collab_emit_kernel(
    const uint16_t* __restrict__ feats, int64_t row_stride, int64_t batch_stride,
    const int32_t* __restrict__ elite, const int32_t* __restrict__ assign,
    const int32_t* __restrict__ out_index, const int32_t* __restrict__ n_out, int n, int D,
    uint16_t* __restrict__ out_feats) {
    const int r = blockIdx.x, b = blockIdx.y;
    if (r >= n_out[b]) return;
    feats += b * batch_stride;
    elite += (int64_t)b * n;
    assign += (int64_t)b * n;
    uint16_t* dst = out_feats + ((int64_t)b * n + r) * D;
    const int first = out_index[(int64_t)b * n + r];
    if (elite[first]) {                                   // an elite row: plain copy
        const uint16_t* src = feats + (int64_t)first * row_stride;
        for (int c = threadIdx.x * 8; c < D; c += 256 * 8)
            *reinterpret_cast<uint4*>(dst + c) = *reinterpret_cast<const uint4*>(src + c);
        return;
    }
    // a merged row: list the absorbed tokens in ascending order (block-wide ordered compaction of
    // the tokens assigned to this row), then average them channel by channel
    __shared__ int members[VITCOP_VIC_MAX_TOKENS];
    __shared__ int wave_tot[4];
    __shared__ int total;
    const int tid = threadIdx.x;
    const int running = block_exclusive_scan<256>(
        first, n, wave_tot, [&](int i) { return assign[i] == r ? 1 : 0; },
        [&](int i, int f, int pos) {
            if (f) members[pos] = i;
        });
    if (tid == 0) total = running;
    __syncthreads();
    const int count = total;
    const float inv = 1.0f / (float)count;
    for (int c = tid * 8; c < D; c += 256 * 8) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int m = 0; m < count; ++m) {
            const uint4 u = *reinterpret_cast<const uint4*>(feats + (int64_t)members[m] * row_stride + c);
            acc[0] += bf16_lo(u.x); acc[1] += bf16_hi(u.x);
            acc[2] += bf16_lo(u.y); acc[3] += bf16_hi(u.y);
            acc[4] += bf16_lo(u.z); acc[5] += bf16_hi(u.z);
            acc[6] += bf16_lo(u.w); acc[7] += bf16_hi(u.w);
        }
        uint4 o;
        o.x = pack_bf16(acc[0] * inv, acc[1] * inv);
        o.y = pack_bf16(acc[2] * inv, acc[3] * inv);
        o.z = pack_bf16(acc[4] * inv, acc[5] * inv);
        o.w = pack_bf16(acc[6] * inv, acc[7] * inv);
        *reinterpret_cast<uint4*>(dst + c) = o;
    }
}

size_t collab_workspace_bytes(int B, int n) { return 2 * up256((size_t)B * n * 4); }   // elite flags, row of every token

int launch_collab(const uint16_t* feats, int64_t row_stride, int64_t batch_stride, const int32_t* labels,
                  const int32_t* n_clusters, const float* norms, int B, int n, int D, int budget,
                  uint16_t* out_feats, int32_t* out_index, int32_t* n_out, int32_t* assign, void* ws,
                  hipStream_t s) {
    if (B == 0) return VITCOP_OK;
    int32_t* elite = static_cast<int32_t*>(ws);
    if (!assign) assign = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + up256((size_t)B * n * 4));
    if (n > 0) {
        dim3 grid((unsigned)((n + CB_ROW_THREADS / 64 - 1) / (CB_ROW_THREADS / 64)), B);
        hipLaunchKernelGGL(collab_rank_kernel, grid, dim3(CB_ROW_THREADS), 0, s, labels, norms, n_clusters, n, budget,
                           elite);
        int rc = launch_status("collab_rank");
        if (rc) return rc;
    }
    static std::atomic<bool> attr_set{false};   // set once; a second thread repeating the call is harmless
    if (!attr_set.load(std::memory_order_acquire)) {
        int rc = hip_status(hipFuncSetAttribute((const void*)collab_plan_kernel,
                                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                                2 * VITCOP_VIC_MAX_TOKENS * 4 + 16),
                            "hipFuncSetAttribute(collab_plan)");
        if (rc) return rc;
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(collab_plan_kernel, dim3(B), dim3(CB_PLAN_THREADS), (size_t)2 * n * 4 + 16, s, labels, elite,
                       n_clusters, n, assign, out_index, n_out);
    int rc = launch_status("collab_plan");
    if (rc || n == 0) return rc;
    hipLaunchKernelGGL(collab_emit_kernel, dim3(n, B), dim3(256), 0, s, feats, row_stride, batch_stride, elite, assign,
                       out_index, n_out, n, D, out_feats);
    return launch_status("collab_emit");
}

}  // namespace vitcop
