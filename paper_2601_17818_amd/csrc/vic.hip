// Visual Information Clustering (Sec. 3.2.1, Eq. 2-3; Alg. 2 of arXiv 2601.17818): a
// density-peak clustering of the visual tokens that survived Stage I, constrained to
// spatial neighbours.
//
//   1. squared row norms of the features                       rowsq_kernel
//   2. D_feat[i,j] = ||f_i - f_j||_2 from an MFMA Gram product  gemm_kernel<.., GM_EPI_DIST>
//   3. rho_i = sum_{j != i} exp(-(D_feat[i,j]/d_c)^2)  (Eq. 2)  vic_density_kernel
//   4. delta_i, N_i = min / argmin of D_feat[i,j] over j with rho_j > rho_i and
//      D_spatial[i,j] <= tau (Eq. 3), gamma_i = rho_i delta_i   vic_parent_kernel
//   5. the n_centers largest gamma are centres; every other token follows its
//      parent pointers N_i up to a root (a centre, or a token without parent);
//      clusters are numbered by the index of their root          vic_label_kernel
//
// Every decision (rho_j > rho_i, the minimum, the TopK of gamma) is taken on the fp32
// values this code writes out, ties going to the lower index, so the result is
// a deterministic function of those arrays.  The order of Step 4 of Alg. 2
// (tokens in decreasing density take their parent's label) is replaced by
// pointer jumping, which reaches the same labels: a parent is strictly denser
// than its child, so the parent chains have no cycles.
#include <atomic>
#include "vitcop_internal.h"
#include "device_utils.h"
#include "select_device.h"

namespace vitcop {

constexpr int VIC_ROW_THREADS = 256;      // 4 wavefronts, one matrix row each

// sq[i] = sum_c f[i,c]^2 in fp32; D % 8 == 0, rows 16-byte aligned
__global__ __launch_bounds__(VIC_ROW_THREADS) void rowsq_kernel(const uint16_t* __restrict__ f,
                                                                int64_t row_stride, int64_t batch_stride,
                                                                int n, int D, float* __restrict__ sq,
                                                                int64_t sq_batch) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * (VIC_ROW_THREADS / 64) + (threadIdx.x >> 6);
    if (i >= n) return;
    sq += blockIdx.y * sq_batch;
    const uint16_t* row = f + blockIdx.y * batch_stride + (int64_t)i * row_stride;
    float acc = 0.f;
    for (int c = lane * 8; c < D; c += 64 * 8) acc = sumsq8(*reinterpret_cast<const uint4*>(row + c), acc);
    acc = wave_sum(acc);
    if (lane == 0) sq[i] = acc;
}

// Eq. 2.  One wavefront per row; lane l adds the columns l, l+64, ... in order, then the 64
// lane sums are combined by the fixed xor tree: the result does not depend on scheduling.
__global__ __launch_bounds__(VIC_ROW_THREADS) void vic_density_kernel(float* __restrict__ dist,
                                                                      int64_t dist_stride,
                                                                      int64_t dist_batch, int n,
                                                                      float neg_inv_dc2_log2e,
                                                                      float* __restrict__ rho) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * (VIC_ROW_THREADS / 64) + (threadIdx.x >> 6);
    if (i >= n) return;
    rho += (int64_t)blockIdx.y * n;
    float* row = dist + blockIdx.y * dist_batch + (int64_t)i * dist_stride;
    if (lane == 0) row[i] = 0.f;                        // a token is at distance 0 from itself
    float acc = 0.f;
    for (int j = lane; j < n; j += 64) {
        const float d = row[j];
        const float e = __builtin_amdgcn_exp2f(d * d * neg_inv_dc2_log2e);
        acc += (j != i) ? e : 0.f;
    }
    acc = wave_sum(acc);
    if (lane == 0) rho[i] = acc;
}

// Eq. 3.  One wavefront per row; candidates are ordered by (distance, index).
__global__ __launch_bounds__(VIC_ROW_THREADS) void vic_parent_kernel(
    const float* __restrict__ dist, int64_t dist_stride, int64_t dist_batch,
    const float* __restrict__ pos, const float* __restrict__ rho, int n, float tau2,
    float* __restrict__ delta, int32_t* __restrict__ parent, float* __restrict__ gamma) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * (VIC_ROW_THREADS / 64) + (threadIdx.x >> 6);
    if (i >= n) return;
    const int64_t img = (int64_t)blockIdx.y * n;
    pos += 2 * img;
    rho += img;
    delta += img;
    parent += img;
    gamma += img;
    const float* row = dist + blockIdx.y * dist_batch + (int64_t)i * dist_stride;
    const float rho_i = rho[i], px = pos[2 * i], py = pos[2 * i + 1];
    float best = INFINITY;
    int best_j = 0x7fffffff;
    for (int j = lane; j < n; j += 64) {
        const float dx = pos[2 * j] - px, dy = pos[2 * j + 1] - py;
        const bool ok = rho[j] > rho_i && dx * dx + dy * dy <= tau2;
        const float d = row[j];
        if (ok && d < best) {          // j ascends within a lane: strict "<" keeps the lower index
            best = d;
            best_j = j;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(best, o, 64);
        const int oj = __shfl_xor(best_j, o, 64);
        if (ob < best || (ob == best && oj < best_j)) {
            best = ob;
            best_j = oj;
        }
    }
    if (lane == 0) {
        const bool none = best_j == 0x7fffffff;
        delta[i] = best;                                 // +inf when no candidate
        parent[i] = none ? -1 : best_j;
        gamma[i] = none ? INFINITY : rho_i * best;
    }
}

// Steps 3-4 of Alg. 2 for one image per workgroup.
__global__ __launch_bounds__(SEL_THREADS) void vic_label_kernel(const float* __restrict__ gamma,
                                                                const int32_t* __restrict__ parent,
                                                                int n, int n_centers,
                                                                int32_t* __restrict__ labels,
                                                                int32_t* __restrict__ n_clusters,
                                                                int64_t batch_stride) {
    extern __shared__ __attribute__((aligned(16))) unsigned vic_lds[];
    __shared__ SelectShared sh;
    __shared__ int wave_tot[SEL_THREADS / 64];
    const int tid = threadIdx.x, b = blockIdx.x;
    gamma += b * batch_stride;
    parent += b * batch_stride;
    labels += b * batch_stride;
    unsigned* keys = vic_lds;                          // [n]  order-preserving keys of gamma, later root pointers
    int32_t* chosen = reinterpret_cast<int32_t*>(vic_lds + n);     // [n_centers] centre indices, later cluster ids [n]
    int32_t* cid = reinterpret_cast<int32_t*>(vic_lds + n);        // (reuses `chosen` once the roots are marked)
    unsigned* is_root = vic_lds + 2 * (size_t)n;       // [n]

    // largest gamma first: complement of the bit pattern (gamma >= 0, +inf allowed)
    for (int i = tid; i < n; i += SEL_THREADS) keys[i] = ~__float_as_uint(gamma[i]);
    __syncthreads();
    block_select_emit(keys, n, n_centers, chosen, 0, sh);
    __syncthreads();
    for (int i = tid; i < n; i += SEL_THREADS) is_root[i] = parent[i] < 0 ? 1u : 0u;
    __syncthreads();
    for (int r = tid; r < n_centers; r += SEL_THREADS) is_root[chosen[r]] = 1u;
    __syncthreads();

    // cluster id of a root = number of roots with a lower index (block-wide exclusive scan over
    // chunks of SEL_THREADS tokens), and the pointer every token starts from
    const int running = block_exclusive_scan<SEL_THREADS>(
        0, n, wave_tot, [&](int i) { return (int)is_root[i]; },
        [&](int i, int f, int before) {
            cid[i] = before;
            keys[i] = f ? (unsigned)i : (unsigned)parent[i];
        });
    if (tid == 0) n_clusters[b] = (int32_t)running;

    // pointer jumping: after ceil(log2 n) rounds every pointer is a root
    for (int span = 1; span < n; span <<= 1) {
        for (int i = tid; i < n; i += SEL_THREADS) {
            const unsigned p = keys[i];
            keys[i] = keys[p];          // concurrent updates only move a pointer further up its own chain
        }
        __syncthreads();
    }
    for (int i = tid; i < n; i += SEL_THREADS) labels[i] = cid[keys[i]];
}

size_t vic_workspace_bytes(int B, int n) {
    const size_t n_pad = ((size_t)n + 3) / 4 * 4;
    // per image: distance matrix, squared norms (padded), rho, delta, gamma, parent
    return (size_t)B * (up256(n_pad * n * 4) + up256(n_pad * 4) + 4 * up256((size_t)n * 4));
}

int launch_vic(const uint16_t* feats, int64_t row_stride, int64_t batch_stride, const float* pos, int B,
               int n, int D, float d_c, float tau, int n_centers, int32_t* labels, int32_t* n_clusters,
               float* rho_out, float* delta_out, int32_t* parent_out, float* dist_out, void* ws,
               hipStream_t s) {
    if (B == 0) return VITCOP_OK;
    if (n == 0) {
        hipLaunchKernelGGL(vic_label_kernel, dim3(B), dim3(SEL_THREADS), 16, s, nullptr, nullptr, 0, 0, labels,
                           n_clusters, 0);
        return launch_status("vic_label");
    }
    const int64_t n_pad = ((int64_t)n + 3) / 4 * 4;
    char* p = static_cast<char*>(ws);
    auto take = [&](size_t bytes) {
        char* r = p;
        p += up256(bytes);
        return r;
    };
    float* dist_ws = reinterpret_cast<float*>(take((size_t)B * n_pad * n * 4));
    float* sq = reinterpret_cast<float*>(take((size_t)B * n_pad * 4));
    float* rho_ws = reinterpret_cast<float*>(take((size_t)B * n * 4));
    float* delta_ws = reinterpret_cast<float*>(take((size_t)B * n * 4));
    float* gamma = reinterpret_cast<float*>(take((size_t)B * n * 4));
    int32_t* parent_ws = reinterpret_cast<int32_t*>(take((size_t)B * n * 4));
    float* dist = dist_out ? dist_out : dist_ws;
    float* rho = rho_out ? rho_out : rho_ws;
    float* delta = delta_out ? delta_out : delta_ws;
    int32_t* parent = parent_out ? parent_out : parent_ws;

    const dim3 row_grid((unsigned)((n + VIC_ROW_THREADS / 64 - 1) / (VIC_ROW_THREADS / 64)), B);
    const float c = -1.4426950408889634f / (d_c * d_c);
    const int64_t dist_batch = (int64_t)n * n_pad;
    hipLaunchKernelGGL(rowsq_kernel, row_grid, dim3(VIC_ROW_THREADS), 0, s, feats, row_stride, batch_stride, n, D, sq,
                       n_pad);
    int rc = launch_status("rowsq");
    if (rc) return rc;
    rc = launch_pairwise_dist(feats, row_stride, batch_stride, sq, n_pad, dist, n_pad, dist_batch, n, D, B, s);
    if (rc) return rc;
    hipLaunchKernelGGL(vic_density_kernel, row_grid, dim3(VIC_ROW_THREADS), 0, s, dist, n_pad, dist_batch, n, c, rho);
    rc = launch_status("vic_density");
    if (rc) return rc;
    hipLaunchKernelGGL(vic_parent_kernel, row_grid, dim3(VIC_ROW_THREADS), 0, s, dist, n_pad, dist_batch, pos, rho, n,
                       tau * tau, delta, parent, gamma);
    rc = launch_status("vic_parent");
    if (rc) return rc;
    const size_t lds = (size_t)3 * n * 4 + 16;
    static std::atomic<bool> attr_set{false};   // set once; a second thread repeating the call is harmless
    if (!attr_set.load(std::memory_order_acquire)) {
        rc = hip_status(hipFuncSetAttribute((const void*)vic_label_kernel,
                                            hipFuncAttributeMaxDynamicSharedMemorySize,
                                            3 * VITCOP_VIC_MAX_TOKENS * 4 + 16),
                        "hipFuncSetAttribute(vic_label)");
        if (rc) return rc;
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(vic_label_kernel, dim3(B), dim3(SEL_THREADS), lds, s, gamma, parent, n, n_centers, labels,
                       n_clusters, (int64_t)n);
    return launch_status("vic_label");
}

}  // namespace vitcop
