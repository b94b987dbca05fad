// One decoding step over a (compacted) KV cache: o = softmax(scale K q) V for the new token of
// every sample, the per-token cost that pruning the prefill reduces afterwards (Table 5 of
// arXiv 2601.17818 reports it).  HBM-bound: K and V of the cache are read exactly once.
//
// decode_partial_kernel: a workgroup takes one KV head, all G = Hq/Hkv query heads that share
// it, and one slice of the keys.  A key row (d bf16) is spread over d/8 lanes, 16 bytes each,
// so a wavefront reads 512/d keys per instruction; every lane keeps, for each of the G query
// heads, its 8 query channels, a running maximum, a running sum and 8 output channels (online
// softmax).  The lane groups, then the wavefronts, are merged at the end and one partial
// (max, sum, unnormalised output) per (sample, head, slice) goes to the workspace.
// decode_merge_kernel combines the slices.
#include "vitcop_internal.h"
#include "device_utils.h"

namespace vitcop {

constexpr int DC_THREADS = 256;
constexpr int DC_MAX_G = 8;              // query heads per KV head handled in one pass

template <int D, int G>
__global__ __launch_bounds__(DC_THREADS) void decode_partial_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    float* __restrict__ part_o, float* __restrict__ part_ml, int N, int Hq, int Hkv, int g0,
    float scale_log2e, int keys_per_split, int n_splits, int64_t kv_batch,
    const int32_t* __restrict__ n_cached_samples) {
    constexpr int LPK = D / 8;                       // lanes per key row
    constexpr int KPW = 64 / LPK;                    // keys per wavefront instruction
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int c = lane % LPK, kq = lane / LPK;
    const int group = Hq / Hkv;
    const int h0 = hk * group + g0;                  // first query head of this pass

    float qv[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int h = min(h0 + g, Hq - 1);
        const uint4 u = *reinterpret_cast<const uint4*>(q + ((int64_t)b * Hq + h) * D + 8 * c);
        qv[g][0] = bf16_lo(u.x); qv[g][1] = bf16_hi(u.x); qv[g][2] = bf16_lo(u.y); qv[g][3] = bf16_hi(u.y);
        qv[g][4] = bf16_lo(u.z); qv[g][5] = bf16_hi(u.z); qv[g][6] = bf16_lo(u.w); qv[g][7] = bf16_hi(u.w);
    }
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }
    // caches of different lengths: sample b attends over its n_cached_samples[b] rows and the appended one;
    // slices past them see no live key and hand on an empty partial (max -inf, sum 0)
    const int n_keys = n_cached_samples ? min(max(n_cached_samples[b], 0) + 1, N) : N;
    const int key_begin = split * keys_per_split, key_end = min(n_keys, key_begin + keys_per_split);
    const int64_t row = (int64_t)Hkv * D;
    const uint16_t* kb = k + b * kv_batch + hk * D + 8 * c;      // kv_batch: elements between two samples' caches
    const uint16_t* vb = v + b * kv_batch + hk * D + 8 * c;
    for (int key0 = key_begin + wv * KPW; key0 < key_end; key0 += 4 * KPW) {     // (empty if key_end <= key_begin)
        const int key = key0 + kq;
        const bool live = key < key_end;
        const int kc = min(key, key_end - 1);
        const uint4 ku = ld_nt16(kb + kc * row), vu = ld_nt16(vb + kc * row);
        const float kf[8] = {bf16_lo(ku.x), bf16_hi(ku.x), bf16_lo(ku.y), bf16_hi(ku.y),
                             bf16_lo(ku.z), bf16_hi(ku.z), bf16_lo(ku.w), bf16_hi(ku.w)};
        const float vf[8] = {bf16_lo(vu.x), bf16_hi(vu.x), bf16_lo(vu.y), bf16_hi(vu.y),
                             bf16_lo(vu.z), bf16_hi(vu.z), bf16_lo(vu.w), bf16_hi(vu.w)};
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s = fmaf(qv[g][e], kf[e], s);
#pragma unroll
            for (int o = LPK / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);      // over the lanes of this key
            s = live ? s * scale_log2e : -INFINITY;
            const float m_new = fmaxf(m[g], s);
            // m_new is -inf only while nothing live has been seen: then alpha and p must be 0, not NaN
            const float alpha = m_new == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m[g] - m_new);
            const float p = m_new == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s - m_new);
            m[g] = m_new;
            l[g] = fmaf(l[g], alpha, p);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(acc[g][e], alpha, p * vf[e]);
        }
    }
    // merge the KPW key sub-groups of the wavefront (lanes with the same c), then the wavefronts
    __shared__ float sm[4][DC_MAX_G][2];
    __shared__ float so[4][DC_MAX_G][D];
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int o = LPK; o < 64; o <<= 1) {
            const float mo = __shfl_xor(m[g], o, 64), lo = __shfl_xor(l[g], o, 64);
            const float mn = fmaxf(m[g], mo);
            const float a0 = mn == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m[g] - mn);
            const float a1 = mn == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mo - mn);
            l[g] = l[g] * a0 + lo * a1;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] = acc[g][e] * a0 + __shfl_xor(acc[g][e], o, 64) * a1;
            m[g] = mn;
        }
        if (kq == 0) {
            if (c == 0) {
                sm[wv][g][0] = m[g];
                sm[wv][g][1] = l[g];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) so[wv][g][8 * c + e] = acc[g][e];
        }
    }
    __syncthreads();
    // threads (g, channel) combine the four wavefronts and write the partial of this slice
    for (int idx = threadIdx.x; idx < G * D; idx += DC_THREADS) {
        const int g = idx / D, ch = idx - g * D;
        if (h0 + g >= hk * group + group) continue;          // padding heads of the last pass
        float mn = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mn = fmaxf(mn, sm[w][g][0]);
        float lt = 0.f, ot = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a = mn == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sm[w][g][0] - mn);
            lt += sm[w][g][1] * a;
            ot += so[w][g][ch] * a;
        }
        const int64_t slot = ((int64_t)b * Hq + h0 + g) * n_splits + split;
        part_o[slot * D + ch] = ot;
        if (ch == 0) {
            part_ml[slot * 2] = mn;
            part_ml[slot * 2 + 1] = lt;
        }
    }
}

template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(const float* __restrict__ part_o,
                                                         const float* __restrict__ part_ml, int n_splits,
                                                         uint16_t* __restrict__ out, float* __restrict__ lse) {
    const int64_t bh = blockIdx.x;
    const int ch = threadIdx.x;
    float mn = -INFINITY;
    for (int s = 0; s < n_splits; ++s) mn = fmaxf(mn, part_ml[(bh * n_splits + s) * 2]);
    float lt = 0.f, ot = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const float ms = part_ml[(bh * n_splits + s) * 2];
        const float a = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - mn);
        lt += part_ml[(bh * n_splits + s) * 2 + 1] * a;
        ot += part_o[(bh * n_splits + s) * D + ch] * a;
    }
    const float r = ot / lt;
    // neighbouring channels pair up into one 32-bit store
    const float r1 = __shfl_down(r, 1, 64);
    if ((ch & 1) == 0) *reinterpret_cast<uint32_t*>(out + bh * D + ch) = pack_bf16(r, r1);
    if (lse && ch == 0) lse[bh] = (mn + __builtin_amdgcn_logf(lt)) * 0.6931471805599453f;
}

int decode_splits(int B, int N, int Hkv) {
    // about four workgroups per CU, slices of at least 64 keys
    const long wgs = (long)B * Hkv;
    long s = (1024 + wgs - 1) / wgs;
    const long max_s = (N + 63) / 64;
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    return (int)s;
}

size_t decode_workspace_bytes(int B, int N, int Hq, int Hkv, int d) {
    const size_t s = decode_splits(B, N, Hkv);
    return up256((size_t)B * Hq * s * d * 4) + up256((size_t)B * Hq * s * 2 * 4);
}

template <int D, int G>
static void launch_partial(dim3 grid, hipStream_t s, const uint16_t* q, const uint16_t* k, const uint16_t* v,
                           float* po, float* pml, int N, int Hq, int Hkv, int g0, float sl2, int kps, int ns,
                           int64_t kv_batch, const int32_t* ncs) {
    hipLaunchKernelGGL((decode_partial_kernel<D, G>), grid, dim3(DC_THREADS), 0, s, q, k, v, po, pml, N, Hq, Hkv, g0,
                       sl2, kps, ns, kv_batch, ncs);
}

template <int D>
static int launch_decode_d(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out, float* lse,
                           int B, int N, int Hq, int Hkv, float scale, void* ws, hipStream_t s, int64_t kv_batch,
                           DecodeParts* hand_over, const int32_t* ncs) {
    const int ns = decode_splits(B, N, Hkv);
    const int kps = ((N + ns - 1) / ns + 63) / 64 * 64;
    float* po = static_cast<float*>(ws);
    float* pml = reinterpret_cast<float*>(static_cast<char*>(ws) + up256((size_t)B * Hq * ns * D * 4));
    const float sl2 = scale * 1.4426950408889634f;
    const int group = Hq / Hkv;
    dim3 grid(ns, Hkv, B);
    for (int g0 = 0; g0 < group; g0 += DC_MAX_G) {
        const int g = std::min(DC_MAX_G, group - g0);
        if (g == 1) launch_partial<D, 1>(grid, s, q, k, v, po, pml, N, Hq, Hkv, g0, sl2, kps, ns, kv_batch, ncs);
        else if (g == 2) launch_partial<D, 2>(grid, s, q, k, v, po, pml, N, Hq, Hkv, g0, sl2, kps, ns, kv_batch, ncs);
        else if (g <= 4) launch_partial<D, 4>(grid, s, q, k, v, po, pml, N, Hq, Hkv, g0, sl2, kps, ns, kv_batch, ncs);
        else launch_partial<D, 8>(grid, s, q, k, v, po, pml, N, Hq, Hkv, g0, sl2, kps, ns, kv_batch, ncs);
        int rc = launch_status("decode_partial");
        if (rc) return rc;
    }
    if (hand_over != nullptr && ns <= DECODE_PARTS_MAX_SPLITS) {       // the caller's next kernel combines the slices
        *hand_over = DecodeParts{po, pml, ns};
        return VITCOP_OK;
    }
    if (hand_over != nullptr) *hand_over = DecodeParts{nullptr, nullptr, 0};
    hipLaunchKernelGGL((decode_merge_kernel<D>), dim3((unsigned)(B * Hq)), dim3(D), 0, s, po, pml, ns, out, lse);
    return launch_status("decode_merge");
}

int launch_decode_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out, float* lse, int B,
                       int N, int Hq, int Hkv, int d, float scale, void* ws, hipStream_t s, int64_t kv_batch,
                       DecodeParts* hand_over, const int32_t* n_cached_samples) {
    if (kv_batch == 0) kv_batch = (int64_t)N * Hkv * d;         // dense caches
    if (d == 64)
        return launch_decode_d<64>(q, k, v, out, lse, B, N, Hq, Hkv, scale, ws, s, kv_batch, hand_over,
                                   n_cached_samples);
    return launch_decode_d<128>(q, k, v, out, lse, B, N, Hq, Hkv, scale, ws, s, kv_batch, hand_over,
                                n_cached_samples);
}

}  // namespace vitcop
