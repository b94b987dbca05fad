// Stage I filter (Sec. 3.1, Eq. 1; Alg. 1 Stage I): saliency of each patch =
// attention it receives from [CLS], summed over heads; keep the top-k.
//
// filter_logits_kernel   : streams the keys once.  A wavefront takes a token
//                          row (H*d bf16), each lane multiplies 16-byte chunks
//                          with the matching chunk of q_cls held in registers,
//                          and lanes of the same head are reduced by shuffles:
//                          one logit per (head, token) goes to the workspace.
// filter_finalize_kernel : one workgroup per image: per-head max and
//                          normaliser, head-summed softmax weight per patch,
//                          then the same radix selection as the K-norm path
//                          on complemented keys (largest first).
#include <mutex>

#include "vitcop_internal.h"
#include "device_utils.h"
#include "select_device.h"

namespace vitcop {

constexpr int FL_THREADS = 256;
constexpr int FL_WAVES = FL_THREADS / 64;
constexpr int FL_TOK = 4;   // tokens a wavefront handles together
constexpr int FL_MAX_H = 256;

__device__ __forceinline__ float dot8(const uint4& a, const float (&q)[8]) {
    float s = bf16_lo(a.x) * q[0];
    s = fmaf(bf16_hi(a.x), q[1], s);
    s = fmaf(bf16_lo(a.y), q[2], s);
    s = fmaf(bf16_hi(a.y), q[3], s);
    s = fmaf(bf16_lo(a.z), q[4], s);
    s = fmaf(bf16_hi(a.z), q[5], s);
    s = fmaf(bf16_lo(a.w), q[6], s);
    s = fmaf(bf16_hi(a.w), q[7], s);
    return s;
}

// CPL = ceil((H*d/8) / 64) chunks per lane.  LPH = d/8 lanes share a head.
template <int CPL, int LPH>
__global__ __launch_bounds__(FL_THREADS) void filter_logits_kernel(
    const uint16_t* __restrict__ q_cls, const uint16_t* __restrict__ k, int N1, int H,
    float scale, float* __restrict__ logits) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int chunks = H * LPH;
    const int64_t row_elems = (int64_t)chunks * 8;
    float q[CPL][8];
    bool valid[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int ch = lane + 64 * c;
        valid[c] = ch < chunks;
        uint4 u = make_uint4(0, 0, 0, 0);
        if (valid[c]) u = reinterpret_cast<const uint4*>(q_cls + (int64_t)b * row_elems)[ch];
        q[c][0] = bf16_lo(u.x); q[c][1] = bf16_hi(u.x);
        q[c][2] = bf16_lo(u.y); q[c][3] = bf16_hi(u.y);
        q[c][4] = bf16_lo(u.z); q[c][5] = bf16_hi(u.z);
        q[c][6] = bf16_lo(u.w); q[c][7] = bf16_hi(u.w);
    }
    const int tok0 = (blockIdx.x * FL_WAVES + wv) * FL_TOK;
    if (tok0 >= N1) return;
    const uint16_t* kb = k + (int64_t)b * N1 * row_elems;
    uint4 v[FL_TOK][CPL];
#pragma unroll
    for (int t = 0; t < FL_TOK; ++t) {
        const int tok = min(tok0 + t, N1 - 1);
        const uint4* p = reinterpret_cast<const uint4*>(kb + (int64_t)tok * row_elems);
#pragma unroll
        for (int c = 0; c < CPL; ++c)
            v[t][c] = valid[c] ? ld_nt16(p + lane + 64 * c)
                               : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < FL_TOK; ++t) {
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            float s = dot8(v[t][c], q[c]);
#pragma unroll
            for (int o = 1; o < LPH; o <<= 1) s += __shfl_xor(s, o, 64);
            const int ch = lane + 64 * c;
            if (valid[c] && (lane % LPH) == 0 && tok0 + t < N1)
                logits[((int64_t)b * H + ch / LPH) * N1 + tok0 + t] = s * scale;
        }
    }
}

__global__ __launch_bounds__(SEL_THREADS) void filter_finalize_kernel(
    const float* __restrict__ logits, int N, int H, int keep, float* __restrict__ scores_out,
    int32_t* __restrict__ idx_out) {
    extern __shared__ unsigned sel_keys[];
    __shared__ SelectShared sh;
    __shared__ float head_max[FL_MAX_H], head_inv[FL_MAX_H];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int N1 = N + 1;
    const float* lg = logits + (int64_t)b * H * N1;
    // (the workgroup is alone on its CU and everything it reads is a round trip to L2: a head's row is read
    // once, all of its loads in flight together, and kept in registers for the second pass)
    constexpr int FF_HELD = 16;                    // logits per lane held in registers: rows up to 1024 tokens
    for (int h = wv; h < H; h += SEL_THREADS / 64) {
        const float* row = lg + (int64_t)h * N1;
        float m = -INFINITY, z = 0.f;
        if (N1 <= 64 * FF_HELD) {
            float held[FF_HELD];
#pragma unroll
            for (int j = 0; j < FF_HELD; ++j) {
                const int i = lane + 64 * j;
                held[j] = i < N1 ? row[i] : -INFINITY;
            }
#pragma unroll
            for (int j = 0; j < FF_HELD; ++j) m = fmaxf(m, held[j]);
            m = wave_max(m);
#pragma unroll
            for (int j = 0; j < FF_HELD; ++j)
                if (lane + 64 * j < N1) z += __expf(held[j] - m);
        } else {
            for (int i = lane; i < N1; i += 64) m = fmaxf(m, row[i]);
            m = wave_max(m);
            for (int i = lane; i < N1; i += 64) z += __expf(row[i] - m);
        }
        z = wave_sum(z);
        if (lane == 0) { head_max[h] = m; head_inv[h] = 1.0f / z; }
    }
    __syncthreads();
    for (int i = tid; i < N; i += SEL_THREADS) {
        float s = 0.f;
        int h = 0;
        for (; h + 8 <= H; h += 8) {               // eight heads' logits in flight, added in head order
            float w[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) w[j] = lg[(int64_t)(h + j) * N1 + i + 1];
#pragma unroll
            for (int j = 0; j < 8; ++j) s = fmaf(__expf(w[j] - head_max[h + j]), head_inv[h + j], s);
        }
        for (; h < H; ++h) s = fmaf(__expf(lg[(int64_t)h * N1 + i + 1] - head_max[h]), head_inv[h], s);
        if (scores_out) scores_out[(int64_t)b * N + i] = s;
        sel_keys[i] = ~__float_as_uint(s);         // s >= 0: complement reverses the order
    }
    __syncthreads();
    block_select_emit(sel_keys, N, keep, idx_out + (int64_t)b * keep, 0, sh);
}

int launch_filter(const uint16_t* q_cls, const uint16_t* k, int B, int N, int H, int d,
                  int keep, float scale, float* scores_out, int32_t* idx_out,
                  float* logits_ws, hipStream_t s) {
    if (B == 0) return VITCOP_OK;
    const int N1 = N + 1;
    const int chunks = H * d / 8;
    const int cpl = (chunks + 63) / 64;
    dim3 grid((N1 + FL_WAVES * FL_TOK - 1) / (FL_WAVES * FL_TOK), B);
#define VITCOP_FL(CPL)                                                                         \
    do {                                                                                       \
        if (d == 64)                                                                           \
            hipLaunchKernelGGL((filter_logits_kernel<CPL, 8>), grid, dim3(FL_THREADS), 0, s,   \
                               q_cls, k, N1, H, scale, logits_ws);                             \
        else                                                                                   \
            hipLaunchKernelGGL((filter_logits_kernel<CPL, 16>), grid, dim3(FL_THREADS), 0, s,  \
                               q_cls, k, N1, H, scale, logits_ws);                             \
    } while (0)
    if (cpl == 1) VITCOP_FL(1);
    else if (cpl == 2) VITCOP_FL(2);
    else if (cpl <= 4) VITCOP_FL(4);
    else return fail(VITCOP_EUNSUPPORTED, "filter: H*d = %d exceeds 2048", H * d);
#undef VITCOP_FL
    int rc = launch_status("filter_logits");
    if (rc) return rc;
    const size_t smem = (size_t)(N > 0 ? N : 1) * sizeof(unsigned);
    if (smem > 40 * 1024) {
        rc = hip_status(hipFuncSetAttribute((const void*)filter_finalize_kernel,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem),
                        "hipFuncSetAttribute(filter_finalize)");
        if (rc) return rc;
    }
    hipLaunchKernelGGL(filter_finalize_kernel, dim3(B), dim3(SEL_THREADS), smem, s, logits_ws, N,
                       H, keep, scores_out, idx_out);
    return launch_status("filter_finalize");
}

// ---- scratch for callers that cannot allocate ---------------------------------
// The logits of one call, in device memory that belongs to the library's code object: every GPU the
// library runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[FILTER_STATIC_SCRATCH_BYTES];

constexpr int FILTER_MAX_DEVICES = 64;
static std::mutex scratch_mutex;
static void* scratch_ptr[FILTER_MAX_DEVICES];      // device address of `scratch` on each device, once looked up

// The address of the current device's copy of `scratch` (looked up once per device, with that device
// current; the array's name itself is only a host-side handle and must never reach a kernel).
int filter_static_scratch(float** out) {
    int dev = -1;
    int rc = hip_status(hipGetDevice(&dev), "hipGetDevice");
    if (rc) return rc;
    if (dev < 0 || dev >= FILTER_MAX_DEVICES) return fail(VITCOP_EUNSUPPORTED, "filter_visual_static: device %d", dev);
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        rc = hip_status(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (rc) return rc;
        if (!p) return fail(VITCOP_EHIP, "filter_visual_static: no address for the scratch array");
        scratch_ptr[dev] = p;
    }
    *out = static_cast<float*>(scratch_ptr[dev]);
    return VITCOP_OK;
}

}  // namespace vitcop
