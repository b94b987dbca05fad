// Element-wise and row-wise pieces of a LLaMA-family decoder layer around the pruned prefill
// (the language model of LLaVA-1.5 / LLaVA-NeXT, Sec. 4.1 of arXiv 2601.17818): RMSNorm, rotary
// position embedding with explicit (gathered) positions, and the SiLU gate of the MLP.  All
// three are single passes over their operands (HBM-bound); the matrix products between them
// are the projection kernel's.
#include "vitcop_internal.h"
#include "device_utils.h"

namespace vitcop {

// y = x / sqrt(mean(x^2) + eps) * w.  One wavefront per row; the row is read once and kept in
// registers for D <= 8192 (16 chunks of 8 per lane), otherwise read twice.
constexpr int RN_THREADS = 256;
constexpr int RN_MAX_CHUNKS = 16;

__global__ __launch_bounds__(RN_THREADS) void rmsnorm_kernel(const uint16_t* __restrict__ x, int64_t x_stride,
                                                             const uint16_t* __restrict__ w, float eps,
                                                             uint16_t* __restrict__ y, int64_t y_stride, int M,
                                                             int D) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * (RN_THREADS / 64) + (threadIdx.x >> 6);
    if (m >= M) return;
    const uint16_t* row = x + (int64_t)m * x_stride;
    uint16_t* out = y + (int64_t)m * y_stride;
    const int chunks = D / 8;                                // 16-byte chunks in the row
    u32x4 held[RN_MAX_CHUNKS];           // (a native vector type: arrays of the uint4 struct end up in scratch)
    float acc = 0.f;
    const bool fits = chunks <= 64 * RN_MAX_CHUNKS;
#pragma unroll
    for (int j = 0; j < RN_MAX_CHUNKS; ++j) {
        const int c = lane + 64 * j;
        if (c < chunks) {
            held[j] = *reinterpret_cast<const u32x4*>(row + 8 * c);
            acc = sumsq8(make_uint4(held[j].x, held[j].y, held[j].z, held[j].w), acc);
        }
    }
    for (int c = lane + 64 * RN_MAX_CHUNKS; c < chunks; c += 64)
        acc = sumsq8(*reinterpret_cast<const uint4*>(row + 8 * c), acc);
    acc = wave_sum(acc);
    const float r = __builtin_amdgcn_rsqf(acc / (float)D + eps);
    auto scale8 = [&](const uint4& v, const uint4& g) {
        uint4 o;
        o.x = pack_bf16(bf16_lo(v.x) * r * bf16_lo(g.x), bf16_hi(v.x) * r * bf16_hi(g.x));
        o.y = pack_bf16(bf16_lo(v.y) * r * bf16_lo(g.y), bf16_hi(v.y) * r * bf16_hi(g.y));
        o.z = pack_bf16(bf16_lo(v.z) * r * bf16_lo(g.z), bf16_hi(v.z) * r * bf16_hi(g.z));
        o.w = pack_bf16(bf16_lo(v.w) * r * bf16_lo(g.w), bf16_hi(v.w) * r * bf16_hi(g.w));
        return o;
    };
#pragma unroll
    for (int j = 0; j < RN_MAX_CHUNKS; ++j) {
        const int c = lane + 64 * j;
        if (c < chunks)
            *reinterpret_cast<uint4*>(out + 8 * c) = scale8(make_uint4(held[j].x, held[j].y, held[j].z, held[j].w),
                                                            *reinterpret_cast<const uint4*>(w + 8 * c));
    }
    if (!fits)
        for (int c = lane + 64 * RN_MAX_CHUNKS; c < chunks; c += 64)
            *reinterpret_cast<uint4*>(out + 8 * c) =
                scale8(*reinterpret_cast<const uint4*>(row + 8 * c), *reinterpret_cast<const uint4*>(w + 8 * c));
}

int launch_rmsnorm(const uint16_t* x, int64_t x_stride, const uint16_t* w, float eps, uint16_t* y,
                   int64_t y_stride, int M, int D, hipStream_t s) {
    if (M == 0) return VITCOP_OK;
    hipLaunchKernelGGL(rmsnorm_kernel, dim3((unsigned)((M + RN_THREADS / 64 - 1) / (RN_THREADS / 64))),
                       dim3(RN_THREADS), 0, s, x, x_stride, w, eps, y, y_stride, M, D);
    return launch_status("rmsnorm");
}

// Rotary embedding in place, rotate-half pairing: channel i < d/2 of a head pairs with channel
// i + d/2 and the pair turns by position * theta^(-2i/d).  One thread owns 8 consecutive low
// channels and the 8 high channels they pair with; a token's rows of q and of k are handled by
// the same workgroup so the angles are computed once per (token, channel group).
constexpr int RP_THREADS = 256;

__global__ __launch_bounds__(RP_THREADS) void rope_kernel(uint16_t* __restrict__ q, uint16_t* __restrict__ k,
                                                          const int32_t* __restrict__ positions, int64_t n_tokens,
                                                          int Hq, int Hkv, int d, float neg_log2_theta_2_over_d) {
    const int groups = d / 16;                      // threads per head: 8 low + 8 high channels each
    const int heads = Hq + Hkv;
    const int64_t idx = (int64_t)blockIdx.x * RP_THREADS + threadIdx.x;
    const int64_t per_token = (int64_t)heads * groups;
    const int64_t token = idx / per_token;
    if (token >= n_tokens) return;
    const int rem = (int)(idx - token * per_token);
    const int head = rem / groups, grp = rem - head * groups;
    uint16_t* base = head < Hq ? q + (token * Hq + head) * d : k + (token * Hkv + (head - Hq)) * d;
    const float pos = (float)positions[token];
    uint4 lo = *reinterpret_cast<const uint4*>(base + 8 * grp);
    uint4 hi = *reinterpret_cast<const uint4*>(base + d / 2 + 8 * grp);
    const uint32_t* lw = reinterpret_cast<const uint32_t*>(&lo);
    const uint32_t* hw = reinterpret_cast<const uint32_t*>(&hi);
    uint32_t ol[4], oh[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        float rl[2], rh[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int i = 8 * grp + 2 * p + e;
            const float inv_freq = __builtin_exp2f((float)i * neg_log2_theta_2_over_d);
            float sn, cs;
            sincosf(pos * inv_freq, &sn, &cs);
            const float a = e ? bf16_hi(lw[p]) : bf16_lo(lw[p]);
            const float b = e ? bf16_hi(hw[p]) : bf16_lo(hw[p]);
            rl[e] = a * cs - b * sn;
            rh[e] = b * cs + a * sn;
        }
        ol[p] = pack_bf16(rl[0], rl[1]);
        oh[p] = pack_bf16(rh[0], rh[1]);
    }
    *reinterpret_cast<uint4*>(base + 8 * grp) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
    *reinterpret_cast<uint4*>(base + d / 2 + 8 * grp) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
}

int launch_rope(uint16_t* q, uint16_t* k, const int32_t* positions, int64_t n_tokens, int Hq, int Hkv, int d,
                float theta, hipStream_t s) {
    if (!q) Hq = 0;
    if (!k) Hkv = 0;
    const int64_t threads = n_tokens * (Hq + Hkv) * (d / 16);
    if (threads == 0) return VITCOP_OK;
    const float c = -2.0f * std::log2(theta) / (float)d;
    hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((threads + RP_THREADS - 1) / RP_THREADS)), dim3(RP_THREADS), 0,
                       s, q, k, positions, n_tokens, Hq, Hkv, d, c);
    return launch_status("rope");
}

// The decoding step's variant: one new token per sample.  q is embedded in place; k is embedded on its way
// into the sample's next cache row (k_dst + b * kv_batch, plus rows[b] rows when the samples' caches have
// different lengths) and v is copied into its row, so the append needs no copies of its own.  Threads: per token (Hq + Hkv) * d/16 rotary groups, then Hkv * d/8 chunks of v.
__global__ __launch_bounds__(RP_THREADS) void rope_append_kernel(
    uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int32_t* __restrict__ positions, int n_tokens, int Hq, int Hkv, int d, float neg_log2_theta_2_over_d,
    uint16_t* __restrict__ k_dst, uint16_t* __restrict__ v_dst, int64_t kv_batch,
    const int32_t* __restrict__ rows) {
    const int groups = d / 16;
    const int rot = (Hq + Hkv) * groups, per_token = rot + Hkv * (d / 8);
    const int idx = blockIdx.x * RP_THREADS + threadIdx.x;
    const int token = idx / per_token;
    if (token >= n_tokens) return;
    const int rem = idx - token * per_token;
    const int64_t cache_off = token * kv_batch + (rows ? (int64_t)rows[token] * Hkv * d : 0);
    if (rem >= rot) {                                   // a 16-byte chunk of v
        const int c = rem - rot;
        *reinterpret_cast<uint4*>(v_dst + cache_off + 8 * c) =
            *reinterpret_cast<const uint4*>(v + ((int64_t)token * Hkv * d) + 8 * c);
        return;
    }
    const int head = rem / groups, grp = rem - head * groups;
    const bool is_q = head < Hq;
    const uint16_t* src = is_q ? q + ((int64_t)token * Hq + head) * d : k + ((int64_t)token * Hkv + (head - Hq)) * d;
    uint16_t* dst = is_q ? q + ((int64_t)token * Hq + head) * d : k_dst + cache_off + (head - Hq) * d;
    const float pos = (float)positions[token];
    const uint4 lo = *reinterpret_cast<const uint4*>(src + 8 * grp);
    const uint4 hi = *reinterpret_cast<const uint4*>(src + d / 2 + 8 * grp);
    const uint32_t* lw = reinterpret_cast<const uint32_t*>(&lo);
    const uint32_t* hw = reinterpret_cast<const uint32_t*>(&hi);
    uint32_t ol[4], oh[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        float rl[2], rh[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int i = 8 * grp + 2 * p + e;
            const float inv_freq = __builtin_exp2f((float)i * neg_log2_theta_2_over_d);
            float sn, cs;
            sincosf(pos * inv_freq, &sn, &cs);
            const float a = e ? bf16_hi(lw[p]) : bf16_lo(lw[p]);
            const float b = e ? bf16_hi(hw[p]) : bf16_lo(hw[p]);
            rl[e] = a * cs - b * sn;
            rh[e] = b * cs + a * sn;
        }
        ol[p] = pack_bf16(rl[0], rl[1]);
        oh[p] = pack_bf16(rh[0], rh[1]);
    }
    *reinterpret_cast<uint4*>(dst + 8 * grp) = make_uint4(ol[0], ol[1], ol[2], ol[3]);
    *reinterpret_cast<uint4*>(dst + d / 2 + 8 * grp) = make_uint4(oh[0], oh[1], oh[2], oh[3]);
}

int launch_rope_append(uint16_t* q, const uint16_t* k, const uint16_t* v, const int32_t* positions, int n_tokens,
                       int Hq, int Hkv, int d, float theta, uint16_t* k_dst, uint16_t* v_dst, int64_t kv_batch,
                       hipStream_t s, const int32_t* rows) {
    const int64_t threads = (int64_t)n_tokens * ((Hq + Hkv) * (d / 16) + Hkv * (d / 8));
    if (threads == 0) return VITCOP_OK;
    const float c = -2.0f * std::log2(theta) / (float)d;
    hipLaunchKernelGGL(rope_append_kernel, dim3((unsigned)((threads + RP_THREADS - 1) / RP_THREADS)), dim3(RP_THREADS),
                       0, s, q, k, v, positions, n_tokens, Hq, Hkv, d, c, k_dst, v_dst, kv_batch, rows);
    return launch_status("rope_append");
}

// out = silu(gate) * up, 8 elements per thread
__global__ __launch_bounds__(256) void silu_mul_kernel(const uint16_t* __restrict__ gate,
                                                       const uint16_t* __restrict__ up,
                                                       uint16_t* __restrict__ out, int64_t chunks) {
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= chunks) return;
    const uint4 g = ld_nt16(gate + 8 * c), u = ld_nt16(up + 8 * c);
    auto gated = [](uint32_t gw, uint32_t uw) {
        const float g0 = bf16_lo(gw), g1 = bf16_hi(gw);
        const float s0 = g0 / (1.0f + __expf(-g0)), s1 = g1 / (1.0f + __expf(-g1));
        return pack_bf16(s0 * bf16_lo(uw), s1 * bf16_hi(uw));
    };
    st_nt16(out + 8 * c, make_uint4(gated(g.x, u.x), gated(g.y, u.y), gated(g.z, u.z), gated(g.w, u.w)));
}

int launch_silu_mul(const uint16_t* gate, const uint16_t* up, uint16_t* out, int64_t n_elems, hipStream_t s) {
    const int64_t chunks = n_elems / 8;
    if (chunks == 0) return VITCOP_OK;
    hipLaunchKernelGGL(silu_mul_kernel, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, gate, up, out,
                       chunks);
    return launch_status("silu_mul");
}

}  // namespace vitcop
