// Projections of one to four rows (the new token of each sample in a decoding step, Table 5 of
// arXiv 2601.17818: time per generated token after a pruned prefill).  With so few rows the
// product is a stream over the weights and nothing else: y[b, n] = sum_k x[b, k] W[n, k] reads
// every weight once from HBM and does two flops per element, so the matrix cores have nothing to
// add and the kernel is written for the memory system instead:
//   * every wavefront reads whole rows of W with 16-byte loads, 64 lanes side by side (1 KB per
//     load instruction, whole 128-byte lines), two rows at a time, the loads of the next piece
//     in flight while the current one is multiplied;
//   * x (at most four rows) sits in LDS as bf16 for the whole kernel; with a norm weight the
//     prologue applies RMSNorm to it first, so the norm needs no kernel or pass of its own;
//   * a workgroup (4 or 8 wavefronts, see gv_threads) owns a contiguous range of row pairs and deals the
//     pieces of that range evenly over its wavefronts; a pair cut between two wavefronts is
//     summed through two LDS slots in a fixed order, so results do not depend on timing;
//   * what follows the product runs in the same kernel on the finished sums: the residual add,
//     silu(gate) * up (a pair = the same row of both matrices), or the rotary embedding of q and
//     k (a pair = channels i and i + d/2 of a head) with k and v written straight into their
//     row of the KV cache.
#include "vitcop_internal.h"
#include "device_utils.h"

#include <atomic>
#include <cmath>

namespace vitcop {

enum { GV_EPI_PLAIN = 0, GV_EPI_SILU = 1, GV_EPI_ROPE = 2 };

// Workgroup shape.  One row, fused q/k/v and gate/up launches: 4 wavefronts, three workgroups per CU (12
// wavefronts, each with a piece in flight and the next one requested: more requests in flight than 8 wavefronts
// give, and a finer grain at the end of the launch); measured 7 % faster on the gate/up matrices and 3 % on q/k/v
// than 8 wavefronts in one workgroup per CU, while deeper queues per wavefront (three pieces) measured slower.
// The plain launches keep 8 wavefronts, one workgroup per CU: the output projection's prologue (combining the
// attention slices) is a chain of loads per thread that doubles with half the threads, and the down projection
// gains nothing.  Two to four rows need more registers per wavefront (two fit per SIMD) and more LDS for x.
template <int NB, int EPI> constexpr int gv_threads() { return NB == 1 && EPI != GV_EPI_PLAIN ? 256 : 512; }
template <int NB, int EPI> constexpr int gv_max_wgs() { return NB == 1 && EPI != GV_EPI_PLAIN ? 768 : 256; }
constexpr int GV_KBLK = 512;               // columns a wavefront covers with one 16-byte load per lane
constexpr int GV_U = 4;                    // column blocks per piece
constexpr int GV_MAX_K = 12288;            // x is held in registers across the prologue: GV_MAX_K / 8 chunks per row

struct GvArgs {
    const uint16_t* x;                     // [B][K], row stride x_stride
    int64_t x_stride;
    const uint16_t* ln_w;                  // RMSNorm weight applied to x first, or nullptr
    float eps;
    const uint16_t* w0;                    // plain: W; silu: gate; rope: wq
    const uint16_t* w1;                    // silu: up; rope: wk
    const uint16_t* w2;                    // rope: wv
    int64_t w_stride;
    int K, n_pairs, pairs_q, pairs_r;      // pairs per workgroup: pairs_q, one more for the first pairs_r
    uint16_t* y;                           // plain: [B][N]; silu: activation [B][F]; rope: q [B][Hq*d]
    int64_t y_stride;
    const uint16_t* res;                   // plain: added to the product, or nullptr
    int64_t res_stride;
    uint16_t* k_dst;                       // rope: row of the K cache that receives sample 0's k
    uint16_t* v_dst;
    int64_t kv_batch;                      // elements between two samples' rows
    const int32_t* kv_rows;                // rope: sample b's row lies kv_rows[b] rows further on, or nullptr
    const int32_t* positions;              // rope: [B]
    int Hq, Hkv, d;
    float rope_c;                          // -2 log2(theta) / d
    const float* part_o;                   // x = the combination of a decoding attention's slices (x unused), or
    const float* part_ml;                  // nullptr: part_o [B*heads][n_splits][head_dim], part_ml [..][n_splits][2]
    int n_splits, head_dim;
};

// Eight consecutive channels (from ch0 on) of one head's attention output from its slices, as
// decode_merge_kernel forms them: slice weights 2^(m_s - max m), sum of weighted outputs over the sum of
// weighted sums, rounded to bf16.  The loads of up to eight slices are in flight together.
__device__ __forceinline__ u32x4 gv_merge8(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                           int64_t slot0, int n_splits, int head_dim, int ch0) {
    float mn = -INFINITY, lt = 0.f, ot[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ot[e] = 0.f;
    for (int s = 0; s < n_splits; ++s) mn = fmaxf(mn, part_ml[(slot0 + s) * 2]);
    for (int s0 = 0; s0 < n_splits; s0 += 8) {
        float ms[8], ls[8];
        float4 lo[8], hi[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t slot = slot0 + min(s0 + j, n_splits - 1);         // past the end: read again, not used
            ms[j] = part_ml[slot * 2];
            ls[j] = part_ml[slot * 2 + 1];
            lo[j] = *reinterpret_cast<const float4*>(part_o + slot * head_dim + ch0);
            hi[j] = *reinterpret_cast<const float4*>(part_o + slot * head_dim + ch0 + 4);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (s0 + j >= n_splits) continue;
            const float a = ms[j] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms[j] - mn);
            lt += ls[j] * a;
            ot[0] += lo[j].x * a; ot[1] += lo[j].y * a; ot[2] += lo[j].z * a; ot[3] += lo[j].w * a;
            ot[4] += hi[j].x * a; ot[5] += hi[j].y * a; ot[6] += hi[j].z * a; ot[7] += hi[j].w * a;
        }
    }
    return u32x4{pack_bf16(ot[0] / lt, ot[1] / lt), pack_bf16(ot[2] / lt, ot[3] / lt),
                 pack_bf16(ot[4] / lt, ot[5] / lt), pack_bf16(ot[6] / lt, ot[7] / lt)};
}

// the two weight rows of pair p
template <int EPI>
__device__ __forceinline__ void gv_rows(const GvArgs& a, int p, const uint16_t*& r0, const uint16_t*& r1) {
    if (EPI == GV_EPI_SILU) {
        r0 = a.w0 + (int64_t)p * a.w_stride;
        r1 = a.w1 + (int64_t)p * a.w_stride;
    } else if (EPI == GV_EPI_ROPE) {
        const int half = a.d / 2, pq = a.Hq * half, pk = a.Hkv * half;
        if (p < pq + pk) {
            const uint16_t* w = p < pq ? a.w0 : a.w1;
            const int pp = p < pq ? p : p - pq;
            const int head = pp / half, i = pp - head * half;
            r0 = w + (int64_t)(head * a.d + i) * a.w_stride;
            r1 = r0 + (int64_t)half * a.w_stride;
        } else {
            r0 = a.w2 + (int64_t)(2 * (p - pq - pk)) * a.w_stride;
            r1 = r0 + a.w_stride;
        }
    } else {
        r0 = a.w0 + (int64_t)(2 * p) * a.w_stride;
        r1 = r0 + a.w_stride;
    }
}

// what happens to the two finished sums of pair p for sample b
template <int EPI>
__device__ __forceinline__ void gv_finish(const GvArgs& a, int p, int b, float v0, float v1) {
    if (EPI == GV_EPI_PLAIN) {
        if (a.res) {
            const uint32_t r = *reinterpret_cast<const uint32_t*>(a.res + (int64_t)b * a.res_stride + 2 * p);
            v0 += bf16_lo(r);
            v1 += bf16_hi(r);
        }
        *reinterpret_cast<uint32_t*>(a.y + (int64_t)b * a.y_stride + 2 * p) = pack_bf16(v0, v1);
    } else if (EPI == GV_EPI_SILU) {
        const uint32_t gu = pack_bf16(v0, v1);               // gate and up as the bf16 tensors they would be
        const float g = bf16_lo(gu), u = bf16_hi(gu);
        const float sl = g / (1.0f + __expf(-g));
        a.y[(int64_t)b * a.y_stride + p] = (uint16_t)(pack_bf16(sl * u, 0.f) & 0xFFFFu);
    } else {
        const int half = a.d / 2, pq = a.Hq * half, pk = a.Hkv * half;
        if (p < pq + pk) {
            const bool is_q = p < pq;
            const int pp = is_q ? p : p - pq;
            const int head = pp / half, i = pp - head * half;
            const uint32_t lh = pack_bf16(v0, v1);           // the projection rounded to bf16, then turned
            const float lo = bf16_lo(lh), hi = bf16_hi(lh);
            const float inv_freq = __builtin_exp2f((float)i * a.rope_c);
            float sn, cs;
            sincosf((float)a.positions[b] * inv_freq, &sn, &cs);
            const uint32_t o = pack_bf16(lo * cs - hi * sn, hi * cs + lo * sn);
            const int64_t extra = a.kv_rows ? (int64_t)a.kv_rows[b] * a.Hkv * a.d : 0;
            uint16_t* dst = is_q ? a.y + (int64_t)b * a.y_stride : a.k_dst + (int64_t)b * a.kv_batch + extra;
            dst[head * a.d + i] = (uint16_t)(o & 0xFFFFu);
            dst[head * a.d + i + half] = (uint16_t)(o >> 16);
        } else {
            const int n = 2 * (p - pq - pk);
            const int64_t extra = a.kv_rows ? (int64_t)a.kv_rows[b] * a.Hkv * a.d : 0;
            *reinterpret_cast<uint32_t*>(a.v_dst + (int64_t)b * a.kv_batch + extra + n) = pack_bf16(v0, v1);
        }
    }
}

// LDS: x as bf16 [NB][k_pad] (k_pad = K rounded up to whole pieces, the tail zero), then the sums of
// cut pairs [pairs per workgroup][2 slots][2 rows][NB], then the prologue's per-wavefront sums.
template <int NB, int EPI>
__global__ __launch_bounds__((gv_threads<NB, EPI>())) void gemv_kernel(GvArgs a) {
    constexpr int GV_THREADS = gv_threads<NB, EPI>(), GV_WAVES = GV_THREADS / 64;
    constexpr int GV_HELD = GV_MAX_K / 8 / GV_THREADS;                 // chunks of x per thread and row in the prologue
    extern __shared__ uint4 gv_lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = a.K, kc = K / 8;
    const int KG = (K + GV_KBLK * GV_U - 1) / (GV_KBLK * GV_U);       // pieces per pair
    const int kpc = KG * GV_U * 64;                                    // padded chunks per row of x
    const int pairs_max = a.pairs_q + (a.pairs_r ? 1 : 0);
    uint4* xs = gv_lds;
    float* cut = reinterpret_cast<float*>(gv_lds + NB * kpc);
    float* red = cut + pairs_max * 4 * NB;

    // this workgroup's pairs and this wavefront's pieces of them
    const int wg = blockIdx.x;
    const int my_pairs = a.pairs_q + (wg < a.pairs_r ? 1 : 0);
    const int p_first = wg * a.pairs_q + min(wg, a.pairs_r);
    const int used = min(GV_WAVES, my_pairs);                          // every range at least one whole pair long
    const int items = my_pairs * KG;
    const int t_begin = wv < used ? (int)((int64_t)items * wv / used) : 0;
    const int t_end = wv < used ? (int)((int64_t)items * (wv + 1) / used) : 0;

    u32x4 buf[2][GV_U][2];
    const uint16_t *r0 = nullptr, *r1 = nullptr;
    auto load_piece = [&](u32x4 (&dst)[GV_U][2], int pl, int kg) {
        gv_rows<EPI>(a, p_first + pl, r0, r1);
#pragma unroll
        for (int u = 0; u < GV_U; ++u) {
            int c = (kg * GV_U + u) * 64 + lane;
            c = c < kc ? c : lane;                  // past the row's end: any chunk of the row, times the zeros of x
            dst[u][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(r0 + 8 * c));
            dst[u][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(r1 + 8 * c));
        }
    };
    int pl = 0, kg = 0;
    if (t_begin < t_end) {
        pl = t_begin / KG;
        kg = t_begin - pl * KG;
        load_piece(buf[0], pl, kg);                 // in flight while x is prepared
    }

    // x into LDS, with RMSNorm applied where a norm weight is given
    {
        u32x4 held[NB][GV_HELD];
        float ss[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            ss[b] = 0.f;
#pragma unroll
            for (int j = 0; j < GV_HELD; ++j) {
                const int c = tid + GV_THREADS * j;
                held[b][j] = u32x4{0u, 0u, 0u, 0u};
                if (c < kc) {
                    if (a.part_o != nullptr) {                    // x[b] = attention output, heads side by side
                        const int head = 8 * c / a.head_dim, heads = K / a.head_dim;
                        held[b][j] = gv_merge8(a.part_o, a.part_ml, ((int64_t)b * heads + head) * a.n_splits,
                                               a.n_splits, a.head_dim, 8 * c - head * a.head_dim);
                    } else {
                        held[b][j] = *reinterpret_cast<const u32x4*>(a.x + (int64_t)b * a.x_stride + 8 * c);
                    }
                }
                ss[b] = sumsq8(make_uint4(held[b][j].x, held[b][j].y, held[b][j].z, held[b][j].w), ss[b]);
            }
        }
        if (a.ln_w) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float s = wave_sum(ss[b]);
                if (lane == 0) red[wv * NB + b] = s;
            }
            __syncthreads();
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < GV_WAVES; ++w) s += red[w * NB + b];
                const float r = __builtin_amdgcn_rsqf(s / (float)K + a.eps);
#pragma unroll
                for (int j = 0; j < GV_HELD; ++j) {
                    const int c = tid + GV_THREADS * j;
                    if (c < kc) {
                        const uint4 g = *reinterpret_cast<const uint4*>(a.ln_w + 8 * c);
                        const u32x4 v = held[b][j];
                        held[b][j].x = pack_bf16(bf16_lo(v.x) * r * bf16_lo(g.x), bf16_hi(v.x) * r * bf16_hi(g.x));
                        held[b][j].y = pack_bf16(bf16_lo(v.y) * r * bf16_lo(g.y), bf16_hi(v.y) * r * bf16_hi(g.y));
                        held[b][j].z = pack_bf16(bf16_lo(v.z) * r * bf16_lo(g.z), bf16_hi(v.z) * r * bf16_hi(g.z));
                        held[b][j].w = pack_bf16(bf16_lo(v.w) * r * bf16_lo(g.w), bf16_hi(v.w) * r * bf16_hi(g.w));
                    }
                }
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
#pragma unroll
            for (int j = 0; j < GV_HELD; ++j) {
                const int c = tid + GV_THREADS * j;
                if (c < kc) xs[b * kpc + c] = make_uint4(held[b][j].x, held[b][j].y, held[b][j].z, held[b][j].w);
            }
            for (int c = kc + tid; c < kpc; c += GV_THREADS) xs[b * kpc + c] = make_uint4(0u, 0u, 0u, 0u);
        }
    }
    __syncthreads();

    float acc[2][NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[0][b] = acc[1][b] = 0.f;
    auto multiply = [&](const u32x4 (&src)[GV_U][2], int kgroup) {
#pragma unroll
        for (int u = 0; u < GV_U; ++u) {
            float w[2][8];
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const u32x4 v = src[u][r];
                w[r][0] = bf16_lo(v.x); w[r][1] = bf16_hi(v.x); w[r][2] = bf16_lo(v.y); w[r][3] = bf16_hi(v.y);
                w[r][4] = bf16_lo(v.z); w[r][5] = bf16_hi(v.z); w[r][6] = bf16_lo(v.w); w[r][7] = bf16_hi(v.w);
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint4 xv = xs[b * kpc + (kgroup * GV_U + u) * 64 + lane];
                const float xf[8] = {bf16_lo(xv.x), bf16_hi(xv.x), bf16_lo(xv.y), bf16_hi(xv.y),
                                     bf16_lo(xv.z), bf16_hi(xv.z), bf16_lo(xv.w), bf16_hi(xv.w)};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    acc[0][b] = fmaf(w[0][e], xf[e], acc[0][b]);
                    acc[1][b] = fmaf(w[1][e], xf[e], acc[1][b]);
                }
            }
        }
    };

    // a range that begins inside a pair holds that pair's second part and finishes it after the barrier
    const int pending = (t_begin < t_end && kg != 0) ? pl : -1;
    bool fresh = kg == 0;                            // the running sums began at the pair's first piece
    auto step = [&](const u32x4 (&cur)[GV_U][2], u32x4 (&nxt)[GV_U][2], int t) {
        int npl = pl, nkg = kg + 1;
        if (nkg == KG) {
            nkg = 0;
            ++npl;
        }
        const bool more = t + 1 < t_end;
        if (more) load_piece(nxt, npl, nkg);
        multiply(cur, kg);
        if (kg == KG - 1 || !more) {                 // the pair, or this wavefront's part of it, ends here
            float v0 = 0.f, v1 = 0.f;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float s0 = wave_sum(acc[0][b]), s1 = wave_sum(acc[1][b]);
                if (lane == b) {
                    v0 = s0;
                    v1 = s1;
                }
                acc[0][b] = acc[1][b] = 0.f;
            }
            if (lane < NB) {
                if (fresh && kg == KG - 1) {
                    gv_finish<EPI>(a, p_first + pl, lane, v0, v1);
                } else {
                    float* slot = cut + ((pl * 2 + (fresh ? 0 : 1)) * 2) * NB;
                    slot[lane] = v0;
                    slot[NB + lane] = v1;
                }
            }
            fresh = true;
        }
        pl = npl;
        kg = nkg;
    };
    for (int t = t_begin; t < t_end; t += 2) {
        step(buf[0], buf[1], t);
        if (t + 1 < t_end) step(buf[1], buf[0], t + 1);
    }
    __syncthreads();
    if (pending >= 0 && lane < NB) {
        const float* s = cut + pending * 4 * NB;
        gv_finish<EPI>(a, p_first + pending, lane, s[lane] + s[2 * NB + lane], s[NB + lane] + s[3 * NB + lane]);
    }
}

bool gemv_applies(int B, int K) {
    return B >= 1 && B <= GV_MAX_ROWS && K % 8 == 0 && K >= GV_KBLK && K <= GV_MAX_K;
}

template <int NB, int EPI>
static int launch_gemv_nb(GvArgs& a, hipStream_t s) {
    constexpr int GV_THREADS = gv_threads<NB, EPI>(), GV_WAVES = GV_THREADS / 64;
    const int wgs = max(1, min(gv_max_wgs<NB, EPI>(), a.n_pairs / GV_WAVES));     // at least one row pair per wavefront
    a.pairs_q = a.n_pairs / wgs;
    a.pairs_r = a.n_pairs % wgs;
    const int KG = (a.K + GV_KBLK * GV_U - 1) / (GV_KBLK * GV_U);
    const size_t lds = (size_t)NB * KG * GV_U * 64 * 16 + (size_t)(a.pairs_q + 1) * 4 * NB * 4 + GV_WAVES * NB * 4;
    static std::atomic<size_t> raised_to{65536};     // (per instantiation) dynamic LDS the kernel may use so far
    if (lds > raised_to.load()) {
        const int rc = hip_status(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemv_kernel<NB, EPI>),
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                                  "hipFuncSetAttribute(gemv)");
        if (rc) return rc;
        raised_to.store(lds);
    }
    hipLaunchKernelGGL((gemv_kernel<NB, EPI>), dim3(wgs), dim3(GV_THREADS), lds, s, a);
    return launch_status("gemv");
}

template <int EPI>
static int launch_gemv_epi(GvArgs& a, int B, hipStream_t s) {
    if (a.n_pairs == 0 || B == 0) return VITCOP_OK;
    switch (B) {
        case 1: return launch_gemv_nb<1, EPI>(a, s);
        case 2: return launch_gemv_nb<2, EPI>(a, s);
        case 3: return launch_gemv_nb<3, EPI>(a, s);
        default: return launch_gemv_nb<4, EPI>(a, s);
    }
}

static GvArgs gv_args(const uint16_t* x, int64_t x_stride, const uint16_t* ln_w, float eps, int K) {
    GvArgs a{};
    a.x = x;
    a.x_stride = x_stride;
    a.ln_w = ln_w;
    a.eps = eps;
    a.K = K;
    a.w_stride = K;
    return a;
}

// y[b, :N] = bf16(norm?(x[b]) W^T + res[b]); N even, W [N][K] dense.  With `attn` (and its head_dim), x[b] is the
// output of a decoding attention still in slices (K = heads * head_dim), combined in the prologue.
int launch_gemv(const uint16_t* x, int64_t x_stride, const uint16_t* ln_w, float eps, const uint16_t* w, uint16_t* y,
                int64_t y_stride, const uint16_t* res, int64_t res_stride, int B, int N, int K, hipStream_t s,
                const DecodeParts* attn, int head_dim) {
    GvArgs a = gv_args(x, x_stride, ln_w, eps, K);
    if (attn != nullptr && attn->part_o != nullptr) {            // x comes from the attention's slices
        a.part_o = attn->part_o;
        a.part_ml = attn->part_ml;
        a.n_splits = attn->n_splits;
        a.head_dim = head_dim;
    }
    a.w0 = w;
    a.n_pairs = N / 2;
    a.y = y;
    a.y_stride = y_stride;
    a.res = res;
    a.res_stride = res_stride;
    return launch_gemv_epi<GV_EPI_PLAIN>(a, B, s);
}

// act[b, :F] = bf16(silu(g) * u), g and u the bf16-rounded rows of norm?(x[b]) Wg^T and Wu^T.
int launch_gemv_gated(const uint16_t* x, int64_t x_stride, const uint16_t* ln_w, float eps, const uint16_t* wg,
                      const uint16_t* wu, uint16_t* act, int64_t act_stride, int B, int F, int K, hipStream_t s) {
    GvArgs a = gv_args(x, x_stride, ln_w, eps, K);
    a.w0 = wg;
    a.w1 = wu;
    a.n_pairs = F;
    a.y = act;
    a.y_stride = act_stride;
    return launch_gemv_epi<GV_EPI_SILU>(a, B, s);
}

// q, k, v of one new token per sample from norm?(x[b]): q [B][Hq*d] with the rotary embedding at
// positions[b]; k (embedded) and v go to k_dst / v_dst + b * kv_batch (+ kv_rows[b] rows), the sample's next
// cache row.
int launch_gemv_qkv_rope(const uint16_t* x, int64_t x_stride, const uint16_t* ln_w, float eps, const uint16_t* wq,
                         const uint16_t* wk, const uint16_t* wv, uint16_t* q, uint16_t* k_dst, uint16_t* v_dst,
                         int64_t kv_batch, const int32_t* positions, int B, int Hq, int Hkv, int d, int K, float theta,
                         hipStream_t s, const int32_t* kv_rows) {
    GvArgs a = gv_args(x, x_stride, ln_w, eps, K);
    a.w0 = wq;
    a.w1 = wk;
    a.w2 = wv;
    a.n_pairs = (Hq + 2 * Hkv) * (d / 2);
    a.y = q;
    a.y_stride = (int64_t)Hq * d;
    a.k_dst = k_dst;
    a.v_dst = v_dst;
    a.kv_batch = kv_batch;
    a.kv_rows = kv_rows;
    a.positions = positions;
    a.Hq = Hq;
    a.Hkv = Hkv;
    a.d = d;
    a.rope_c = -2.0f * std::log2(theta) / (float)d;
    return launch_gemv_epi<GV_EPI_ROPE>(a, B, s);
}

}  // namespace vitcop
