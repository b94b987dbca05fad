// Linear projection y = x W^T for FEW rows (M <= 256): what the projections of a decoder layer
// look like after the pruning of Sec. 3.2.2 has cut the sequence to a few hundred tokens.  The
// weight matrix is then nearly all of the traffic (one pass over W per launch) and the launch is
// bound by HBM, not by the matrix cores.  One CU with four wavefronts pulls at most about 50 GB/s
// from HBM, so the whole chip must take part, whatever N and K are:
//
//   * the work is cut into units of (128 output columns) x (64 k-values); the units, ordered
//     column group by column group, are dealt out evenly to at most 256 workgroups, so a
//     workgroup's share is a k-range of one column group, or the tail of one group and the head
//     of the next (two segments);
//   * both operands are fetched with whole 128-byte lines per 8 lanes (the vector memory path
//     moves lines, so the MFMA operand layout, 32 rows x 32 bytes per instruction, would cost four
//     times the cycles) into registers, two units ahead of the multiply, and written to one of
//     two LDS slabs one unit before their use, with the same swizzle as the big-tile GEMM; all
//     loads are ordinary ones, so the compiler's own counting of outstanding loads places every
//     wait (mixed with direct-to-LDS loads it falls back to full drains);
//   * the four wavefronts sit 2 x 2 over the (rows of x) x (128 columns) tile;
//   * up to three weight matrices can sit side by side in one launch (K, Q and V; gate and up);
//   * every segment writes an fp32 partial tile; a second kernel adds the partials of a column
//     group in workgroup order (deterministic) and finishes the rows in one of three ways: residual,
//     bf16 rounding and, for the K projection, the per-128-column sums of squares of the rounded
//     outputs for the K-norm of Eq. 4; the same plus the RMSNorm of the finished row; or the gated
//     activation silu(gate) * up of the MLP.  The same reductions serve the split-K launches of the
//     big-tile kernel (gemm.hip), whose partials are whole slices.
#include <atomic>
#include <cmath>
#include "vitcop_internal.h"
#include "device_utils.h"

namespace vitcop {

constexpr int SK_THREADS = 256;
constexpr int SK_COLS = 128;          // output columns per unit
constexpr int SK_UNIT = 64;           // k-values per unit (one 128-byte line per row)
constexpr int SK_MAX_ROWS = 256;
constexpr int SK_MAX_WGS = 256;       // one per CU

// Units held in registers: the one being stored to LDS and one more in flight behind it.  A deeper
// ring does not put more bytes in flight: a CU's load queue fills, the wavefront blocks on issuing
// the prologue's loads, and the first multiply only starts later (measured with 4, 6 and 8 slots).
constexpr int SK_SLOTS = 2;

struct SkPick {
    int mi, start;
};
__device__ __forceinline__ SkPick sk_pick(const SkMats& mats, int n) {
    const int mi = (n >= mats.n_end[0] ? 1 : 0) + (n >= mats.n_end[1] ? 1 : 0);
    return {mi, mi == 0 ? 0 : (mi == 1 ? mats.n_end[0] : mats.n_end[1])};
}

// Workgroup i of P owns the units [first(i), first(i+1)) of the group-major order: total / P units
// each, one more for the first total % P workgroups (q and r below; no division on the device).
__host__ __device__ __forceinline__ int sk_first_unit(int i, int q, int r) { return i * q + min(i, r); }

// part[2 * workgroup + segment][m][128] (fp32) = sum over the segment's k-range of x[m,k] W[n,k]
// for the 128 columns n of the segment's group.  With part == nullptr every workgroup owns exactly
// one whole column group and writes bf16(sum + residual) to its matrix's output itself.
template <int MB>
__global__ __launch_bounds__(SK_THREADS) void gemm_skinny_kernel(
    const uint16_t* __restrict__ x, int64_t x_stride, SkMats mats, int64_t w_stride, int M, int N, int K,
    int units_q, int units_r, float* __restrict__ part, const uint16_t* __restrict__ res,
    int64_t res_stride) {
    constexpr int NSLOT = SK_SLOTS;
    constexpr int XROWS = MB * 32;
    constexpr int ROWS = XROWS + SK_COLS;                // slab rows: x, then the group's rows of W
    constexpr int SLAB = ROWS * 128;                     // bytes: 64 k-values per row
    constexpr int NLD = ROWS / 8 / 4;                    // loads per wavefront per unit (8 rows each)
    constexpr int MI = MB / 2;                           // row blocks per wavefront (2 x 2 wavefronts: rows x columns)
    constexpr int SROW = 256 + 16;                       // epilogue staging row: 64 fp32, padded
    constexpr int STAGE = 32 * SROW;                     // per wavefront: one 32 x 64 block
    static_assert(NSLOT % 2 == 0, "the slab of a unit must be known at compile time");
    static_assert(MB % 2 == 0, "two wavefronts share the rows");
    static_assert(2 * SLAB >= 4 * STAGE, "the epilogue reuses the slabs");
    extern __shared__ __attribute__((aligned(1024))) char sk_lds[];     // 2 * SLAB bytes

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    // A wavefront multiplies MI row blocks of x with 2 column blocks of W: (MI + 2) fragment reads per
    // 2 MI multiplies; one column block against all rows would read (MB + 1) per MB, and the LDS
    // reads of the four wavefronts are what bounds the loop at 192 and 256 rows.
    const int wr = wv & 1, wc = wv >> 1;
    const int upg = K / SK_UNIT;                         // units per column group
    const int first = sk_first_unit(blockIdx.x, units_q, units_r);
    const int last = sk_first_unit(blockIdx.x + 1, units_q, units_r);    // exclusive; last - first <= upg
    const int m_rows = M;                                // <= MB * 32

    // every wavefront's LDS accesses are done, its writes visible, after this
    auto lds_barrier = [&]() {
        __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0) only: the global loads stay in flight
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    for (int seg = 0, u_begin = first; u_begin < last; ++seg) {
        const int grp = (int)((unsigned)u_begin / (unsigned)upg);
        const int u0 = u_begin - grp * upg;                          // first unit inside the group
        const int nk = min(last, (grp + 1) * upg) - u_begin;         // units of this segment
        u_begin += nk;
        const SkPick pick = sk_pick(mats, grp * SK_COLS);            // which matrix this group belongs to
        const int n0 = grp * SK_COLS - pick.start;                   // first column inside that matrix
        const int n_rows = mats.n_end[pick.mi] - pick.start;
        const uint16_t* wm = mats.w[pick.mi];

        f32x16 acc[MI][2];
#pragma unroll
        for (int j = 0; j < MI; ++j)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

        // Load q of wavefront wv covers slab rows (wv*NLD+q)*8 .. +8; lane L fetches chunk L%8 (16
        // bytes) of row L/8 and stores it at chunk position (L%8) ^ (row%8).
        // (operand base in scalar registers + a 32-bit lane offset: operands are below 2^31 elements;
        // whether a load fetches x or W is uniform, so stride, row limit and row shift are picked as
        // scalars first: a workgroup starts with one wavefront per SIMD, which issues an instruction
        // every few cycles, so every instruction ahead of the first load delays the whole launch)
        const char* base[NLD];
        unsigned src[NLD];
        int dst[NLD];
        const int xs32 = (int)x_stride, ws32 = (int)w_stride;
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            const int row0 = (wv * NLD + q) * 8, row = row0 + (lane >> 3);
            const bool is_x = row0 < XROWS;                          // uniform: 8 rows never straddle
            base[q] = reinterpret_cast<const char*>(is_x ? x : wm);
            const int stride = is_x ? xs32 : ws32, limit = is_x ? m_rows - 1 : n_rows - 1;
            const int shift = is_x ? 0 : n0 - XROWS;
            src[q] = 2u * (unsigned)(min(row + shift, limit) * stride) + 16 * (lane & 7);
            dst[q] = row * 128 + (((lane & 7) ^ (row & 7)) << 4);
        }
        u32x4 held[NSLOT][NLD];
        // Past the segment's end every lane reads the operand's first 16 bytes instead (one line per
        // instruction, never used): the number of loads in flight stays a compile-time fact, which
        // the compiler's wait counts need, while the memory pipeline carries next to nothing for
        // them; with a handful of units per segment, full loads that nobody uses would be a large
        // part of its work.
        auto issue_loads = [&](int slot, int step) {
            const bool live = step < nk;
            const int64_t off = live ? (int64_t)(u0 + step) * (SK_UNIT * 2) : 0;
#pragma unroll
            for (int q = 0; q < NLD; ++q)
                held[slot][q] = *reinterpret_cast<const u32x4*>(base[q] + off + (live ? src[q] : 0u));
        };
        auto store_slab = [&](int slot, int slab) {
#pragma unroll
            for (int q = 0; q < NLD; ++q) *reinterpret_cast<u32x4*>(sk_lds + slab * SLAB + dst[q]) = held[slot][q];
        };
        // MFMA fragments: lane (l32, g) reads the 8 k-values 16*kc + 8*g .. of a row
        bf16x8 xf[2][MI], wf[2][2];
        auto read_frags = [&](int buf, int slab, int kc) {
            const char* S = sk_lds + slab * SLAB;
#pragma unroll
            for (int j = 0; j < MI; ++j) {
                const int row = (wr * MI + j) * 32 + l32;
                xf[buf][j] = *reinterpret_cast<const bf16x8*>(S + row * 128 + (((2 * kc + g) ^ (row & 7)) << 4));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = XROWS + (wc * 2 + i) * 32 + l32;
                wf[buf][i] = *reinterpret_cast<const bf16x8*>(S + row * 128 + (((2 * kc + g) ^ (row & 7)) << 4));
            }
        };
        auto multiply = [&](int buf) {
#pragma unroll
            for (int j = 0; j < MI; ++j)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][i], xf[buf][j], acc[j][i], 0, 0, 0);
        };
        // Scheduling hints: a phase is MB multiplies; the MI + 2 LDS reads of the next phase's
        // fragments follow the first multiplies one by one and, if `extra` names a class (0x200 LDS
        // write, 0x020 global load), every multiply is followed by one instruction of that class;
        // what is left of the NLD extras closes the phase.
#define VITCOP_PHASE(extra)                                              \
    _Pragma("unroll") for (int q_ = 0; q_ < MB; ++q_) {                  \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);               \
        if (q_ < MI + 2) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); \
        if ((extra) != 0) __builtin_amdgcn_sched_group_barrier((extra), 1, 0); \
    }                                                                    \
    if (MB < MI + 2) __builtin_amdgcn_sched_group_barrier(0x100, MI + 2 - MB, 0); \
    if ((extra) != 0) __builtin_amdgcn_sched_group_barrier((extra), NLD - MB, 0);
        // Unit t: slab t % 2, registers slot t % NSLOT.  The operands of unit t+1 go to the other
        // slab (every wavefront left it at the barrier that ended unit t-1); the loads of unit
        // t+1+NSLOT take the registers just stored.  The fragments of a 16-wide slice are read
        // while the slice before it is multiplied.
        auto unit = [&](int t, int slot) {
            const int slab = slot & 1, next = (slot + 1) % NSLOT;
            read_frags(1, slab, 1);               // reads before writes: the compiler keeps LDS accesses in order
            store_slab(next, slab ^ 1);
            multiply(0);
            VITCOP_PHASE(0x200)
            issue_loads(next, t + 1 + NSLOT);
            read_frags(0, slab, 2);
            multiply(1);
            VITCOP_PHASE(0x020)
            read_frags(1, slab, 3);
            multiply(0);
            VITCOP_PHASE(0)
            lds_barrier();
            read_frags(0, slab ^ 1, 0);
            multiply(1);
            VITCOP_PHASE(0)
        };
        // The wavefronts issue their first loads unit by unit in step (a barrier between units):
        // left alone, the oldest wavefront queues all of its loads first and the unit-0 data of
        // the youngest, which the first barrier of the pipeline waits for, arrives last.
        lds_barrier();                            // the slabs are free (previous segment's epilogue)
#pragma unroll
        for (int p = 0; p < NSLOT; ++p) {
            issue_loads(p, p);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        store_slab(0, 0);
        issue_loads(0, NSLOT);
        lds_barrier();
        read_frags(0, 0, 0);
        int t = 0;
        for (; t + NSLOT <= nk; t += NSLOT) {
#pragma unroll
            for (int p = 0; p < NSLOT; ++p) unit(t + p, p);
        }
#pragma unroll
        for (int p = 0; p < NSLOT - 1; ++p)
            if (t + p < nk) unit(t + p, p);
#undef VITCOP_PHASE

        // Epilogue.  A lane owns row m = 32 j + l32 and the column runs n = 8 (r/4) + 4 g + r%4 of
        // its wavefront's 32: stored from there, an instruction would touch 32 rows with 32 bytes
        // each.  Each wavefront stages one 32 x 64 block at a time in LDS (rows padded by 16 bytes)
        // and writes it with 16 lanes per 256-byte row piece of the partial tile.
        lds_barrier();                                       // the last unit's slab reads are done
        char* stage = sk_lds + wv * STAGE;
        const int srow = lane >> 4, scol = (lane & 15) * 4;  // store side: row within a group of 4, first column
        const int n = n0 + wc * 64 + scol;                   // column inside the selected matrix
        const int m0 = wr * MI * 32;                         // first row of this wavefront
        // running addresses, 4 rows further per store (kept as additions: what the compiler hoists
        // to the top of the kernel from here runs ahead of the first load)
        float* out = part + ((int64_t)(2 * blockIdx.x + seg) * M + m0 + srow) * SK_COLS + wc * 64 + scol;
        const int64_t y_stride = mats.y_stride[pick.mi];
        uint16_t* yrow = mats.y[pick.mi] + (int64_t)(m0 + srow) * y_stride + n;
        const uint16_t* rrow = res + (int64_t)(m0 + srow) * res_stride + n;
#pragma unroll
        for (int j = 0; j < MI; ++j) {
            if (m0 + j * 32 >= m_rows) break;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    float4 o;
                    o.x = acc[j][i][4 * r4];
                    o.y = acc[j][i][4 * r4 + 1];
                    o.z = acc[j][i][4 * r4 + 2];
                    o.w = acc[j][i][4 * r4 + 3];
                    *reinterpret_cast<float4*>(stage + l32 * SROW + (32 * i + 8 * r4 + 4 * g) * 4) = o;
                }
            // (a wavefront reads back only what it wrote itself: the LDS counter suffices, no barrier)
#pragma unroll
            for (int r0 = 0; r0 < 32; r0 += 4) {
                const int m = m0 + j * 32 + r0 + srow;
                float4 o = *reinterpret_cast<const float4*>(stage + (r0 + srow) * SROW + scol * 4);
                if (m < m_rows) {
                    if (part != nullptr) {
                        *reinterpret_cast<float4*>(out) = o;
                    } else if (n < n_rows) {                         // direct: the segment is the whole k-range
                        if (res) {
                            const uint2 rr = *reinterpret_cast<const uint2*>(rrow);
                            o.x += bf16_lo(rr.x); o.y += bf16_hi(rr.x);
                            o.z += bf16_lo(rr.y); o.w += bf16_hi(rr.y);
                        }
                        uint2 pk;
                        pk.x = pack_bf16(o.x, o.y);
                        pk.y = pack_bf16(o.z, o.w);
                        *reinterpret_cast<uint2*>(yrow) = pk;
                    }
                }
                out += 4 * SK_COLS;
                yrow += 4 * y_stride;
                rrow += 4 * res_stride;
            }
        }
    }
}

// v[0..8) = sum, in workgroup (or slice) order, of the partials of row m, columns n .. n+8 (n a
// multiple of 8).  Four loads are in flight at a time; the additions keep the order.
__device__ __forceinline__ void sk_sum_tiles(const SkParts& P, int m, int n, float (&v)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.f;
    auto sum_range = [&](int i, int i_hi, auto tile) {
        for (; i + 3 <= i_hi; i += 4) {
            float4 a[4], b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float* p = tile(i + t);
                a[t] = *reinterpret_cast<const float4*>(p);
                b[t] = *reinterpret_cast<const float4*>(p + 4);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                v[0] += a[t].x; v[1] += a[t].y; v[2] += a[t].z; v[3] += a[t].w;
                v[4] += b[t].x; v[5] += b[t].y; v[6] += b[t].z; v[7] += b[t].w;
            }
        }
        for (; i <= i_hi; ++i) {
            const float* p = tile(i);
            const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
            v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
            v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
        }
    };
    if (P.units_q == 0) {
        sum_range(0, P.units_r - 1, [&](int sl) { return P.part + ((int64_t)sl * P.M + m) * P.upg + n; });
        return;
    }
    const int grp = n / SK_COLS;
    auto owner = [&](int u) {               // the workgroup whose unit range holds unit u
        const int big = P.units_r * (P.units_q + 1);      // units held by the workgroups with one more
        return u < big ? u / (P.units_q + 1) : P.units_r + (u - big) / P.units_q;
    };
    sum_range(owner(grp * P.upg), owner((grp + 1) * P.upg - 1), [&](int i) {
        const int seg = sk_first_unit(i, P.units_q, P.units_r) / P.upg == grp ? 0 : 1;   // its first or its second group
        return P.part + ((int64_t)(2 * i + seg) * P.M + m) * SK_COLS + (n & (SK_COLS - 1));
    });
}

// The same for two column chunks of one 128-column group at once, n .. n+8 and n+delta .. n+delta+8: both
// chunks' loads of four tiles are in flight together.
__device__ __forceinline__ void sk_sum_tiles2(const SkParts& P, int m, int n, int delta, float (&v)[8], float (&w)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = w[e] = 0.f;
    auto sum_range = [&](int i, int i_hi, auto tile) {
        for (; i + 3 <= i_hi; i += 4) {
            float4 a[4], b[4], c[4], d[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float* p = tile(i + t);
                a[t] = *reinterpret_cast<const float4*>(p);
                b[t] = *reinterpret_cast<const float4*>(p + 4);
                c[t] = *reinterpret_cast<const float4*>(p + delta);
                d[t] = *reinterpret_cast<const float4*>(p + delta + 4);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                v[0] += a[t].x; v[1] += a[t].y; v[2] += a[t].z; v[3] += a[t].w;
                v[4] += b[t].x; v[5] += b[t].y; v[6] += b[t].z; v[7] += b[t].w;
                w[0] += c[t].x; w[1] += c[t].y; w[2] += c[t].z; w[3] += c[t].w;
                w[4] += d[t].x; w[5] += d[t].y; w[6] += d[t].z; w[7] += d[t].w;
            }
        }
        for (; i <= i_hi; ++i) {
            const float* p = tile(i);
            const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
            const float4 c = *reinterpret_cast<const float4*>(p + delta), d = *reinterpret_cast<const float4*>(p + delta + 4);
            v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
            v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
            w[0] += c.x; w[1] += c.y; w[2] += c.z; w[3] += c.w;
            w[4] += d.x; w[5] += d.y; w[6] += d.z; w[7] += d.w;
        }
    };
    if (P.units_q == 0) {
        sum_range(0, P.units_r - 1, [&](int sl) { return P.part + ((int64_t)sl * P.M + m) * P.upg + n; });
        return;
    }
    const int grp = n / SK_COLS;
    auto owner = [&](int u) {
        const int big = P.units_r * (P.units_q + 1);
        return u < big ? u / (P.units_q + 1) : P.units_r + (u - big) / P.units_q;
    };
    sum_range(owner(grp * P.upg), owner((grp + 1) * P.upg - 1), [&](int i) {
        const int seg = sk_first_unit(i, P.units_q, P.units_r) / P.upg == grp ? 0 : 1;
        return P.part + ((int64_t)(2 * i + seg) * P.M + m) * SK_COLS + (n & (SK_COLS - 1));
    });
}

// y[m, n..n+8) = bf16(sum of the partial tiles of n's column group, in workgroup order, + residual);
// one thread per 8 columns, 16 consecutive lanes per 128-column group, which also yields that
// group's sum of squares of the rounded outputs.  P = workgroups of the first kernel.
__global__ __launch_bounds__(256) void gemm_skinny_reduce_kernel(
    SkParts parts, int N, SkMats mats, const uint16_t* __restrict__ res, int64_t res_stride,
    float* __restrict__ sumsq_parts) {
    const int M = parts.M;
    const int groups = (N + SK_COLS - 1) / SK_COLS, chunks = groups * 16;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int m = (int)(id / chunks), c = (int)(id % chunks);
    const int n = c * 8, grp = c >> 4;
    float ss = 0.f;
    if (m < M && n < N) {
        float v[8];
        sk_sum_tiles(parts, m, n, v);
        const SkPick pick = sk_pick(mats, n);
        uint16_t* dst = mats.y[pick.mi] + (int64_t)m * mats.y_stride[pick.mi] + (n - pick.start);
        if (res) {
            const uint4 r = *reinterpret_cast<const uint4*>(res + (int64_t)m * res_stride + n);
            v[0] += bf16_lo(r.x); v[1] += bf16_hi(r.x);
            v[2] += bf16_lo(r.y); v[3] += bf16_hi(r.y);
            v[4] += bf16_lo(r.z); v[5] += bf16_hi(r.z);
            v[6] += bf16_lo(r.w); v[7] += bf16_hi(r.w);
        }
        uint4 o;
        o.x = pack_bf16(v[0], v[1]);
        o.y = pack_bf16(v[2], v[3]);
        o.z = pack_bf16(v[4], v[5]);
        o.w = pack_bf16(v[6], v[7]);
        *reinterpret_cast<uint4*>(dst) = o;
        if (sumsq_parts) {
            float a;
            a = bf16_lo(o.x); ss = fmaf(a, a, ss);
            a = bf16_hi(o.x); ss = fmaf(a, a, ss);
            a = bf16_lo(o.y); ss = fmaf(a, a, ss);
            a = bf16_hi(o.y); ss = fmaf(a, a, ss);
            a = bf16_lo(o.z); ss = fmaf(a, a, ss);
            a = bf16_hi(o.z); ss = fmaf(a, a, ss);
            a = bf16_lo(o.w); ss = fmaf(a, a, ss);
            a = bf16_hi(o.w); ss = fmaf(a, a, ss);
        }
    }
    if (sumsq_parts) {                                   // uniform branch: every lane takes part in the shuffles
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
        if ((c & 15) == 0 && m < M && n < N) sumsq_parts[(int64_t)grp * M + m] = ss;
    }
}

// Workgroups of the first kernel: one per CU if there is work for that many (two units each at
// least), never fewer than column groups (so that a workgroup's share stays within two groups).
// The same reduction followed by an RMSNorm of the finished row (the next operation of a decoder
// layer after its attention and MLP output projections): y as above, and
// norm_out[m, :] = y[m, :] / sqrt(mean(y[m, :]^2) + eps) * ln_w, computed from the ROUNDED y exactly as
// rmsnorm_kernel does.  One workgroup per row; a thread owns the chunks tid, tid + 256, ...
// (N <= 8 * 256 * SK_NORM_CHUNKS).
constexpr int SK_NORM_CHUNKS = 16;

__global__ __launch_bounds__(256) void gemm_skinny_reduce_norm_kernel(
    SkParts parts, int N, uint16_t* __restrict__ y, int64_t y_stride, const uint16_t* __restrict__ res,
    int64_t res_stride, const uint16_t* __restrict__ ln_w, float eps, uint16_t* __restrict__ norm_out,
    int64_t norm_stride) {
    __shared__ float wave_part[4];
    const int m = blockIdx.x, tid = threadIdx.x;
    const int chunks = N / 8;
    u32x4 held[SK_NORM_CHUNKS];          // (a native vector type: arrays of the uint4 struct end up in scratch)
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < SK_NORM_CHUNKS; ++j) {
        const int c = tid + 256 * j;
        if (c >= chunks) break;
        const int n = c * 8;
        float v[8];
        sk_sum_tiles(parts, m, n, v);
        if (res) {
            const uint4 r = *reinterpret_cast<const uint4*>(res + (int64_t)m * res_stride + n);
            v[0] += bf16_lo(r.x); v[1] += bf16_hi(r.x);
            v[2] += bf16_lo(r.y); v[3] += bf16_hi(r.y);
            v[4] += bf16_lo(r.z); v[5] += bf16_hi(r.z);
            v[6] += bf16_lo(r.w); v[7] += bf16_hi(r.w);
        }
        uint4 o;
        o.x = pack_bf16(v[0], v[1]);
        o.y = pack_bf16(v[2], v[3]);
        o.z = pack_bf16(v[4], v[5]);
        o.w = pack_bf16(v[6], v[7]);
        *reinterpret_cast<uint4*>(y + (int64_t)m * y_stride + n) = o;
        held[j] = u32x4{o.x, o.y, o.z, o.w};
        ss = sumsq8(o, ss);
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) wave_part[tid >> 6] = ss;
    __syncthreads();
    ss = (wave_part[0] + wave_part[1]) + (wave_part[2] + wave_part[3]);
    const float r = __builtin_amdgcn_rsqf(ss / (float)N + eps);
#pragma unroll
    for (int j = 0; j < SK_NORM_CHUNKS; ++j) {
        const int c = tid + 256 * j;
        if (c >= chunks) break;
        const uint4 v = make_uint4(held[j].x, held[j].y, held[j].z, held[j].w);
        const uint4 g = *reinterpret_cast<const uint4*>(ln_w + 8 * c);
        uint4 o;
        o.x = pack_bf16(bf16_lo(v.x) * r * bf16_lo(g.x), bf16_hi(v.x) * r * bf16_hi(g.x));
        o.y = pack_bf16(bf16_lo(v.y) * r * bf16_lo(g.y), bf16_hi(v.y) * r * bf16_hi(g.y));
        o.z = pack_bf16(bf16_lo(v.z) * r * bf16_lo(g.z), bf16_hi(v.z) * r * bf16_hi(g.z));
        o.w = pack_bf16(bf16_lo(v.w) * r * bf16_lo(g.w), bf16_hi(v.w) * r * bf16_hi(g.w));
        *reinterpret_cast<uint4*>(norm_out + (int64_t)m * norm_stride + 8 * c) = o;
    }
}

// The reduction of a gate/up pair launch (columns [0, F) gate, [F, 2F) up) followed by the gated
// activation of the MLP: out[m, n] = bf16(silu(g) * u) with g and u the bf16-rounded projections,
// exactly what silu_mul_kernel computes from stored gate and up tensors.  One thread per 8 columns.
__global__ __launch_bounds__(256) void gemm_skinny_reduce_silu_kernel(
    SkParts parts, int F, uint16_t* __restrict__ out, int64_t out_stride) {
    const int chunks = F / 8, M = parts.M;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int m = (int)(id / chunks), c = (int)(id % chunks);
    if (m >= M) return;
    // bf16(sum of the partial tiles of the 8 columns from n on, in workgroup order), packed
    auto reduced = [&](int n) {
        float v[8];
        sk_sum_tiles(parts, m, n, v);
        return make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
    };
    const uint4 g = reduced(8 * c), u = reduced(F + 8 * c);
    auto gated = [](uint32_t gw, uint32_t uw) {
        const float g0 = bf16_lo(gw), g1 = bf16_hi(gw);
        const float s0 = g0 / (1.0f + __expf(-g0)), s1 = g1 / (1.0f + __expf(-g1));
        return pack_bf16(s0 * bf16_lo(uw), s1 * bf16_hi(uw));
    };
    *reinterpret_cast<uint4*>(out + (int64_t)m * out_stride + 8 * c) =
        make_uint4(gated(g.x, u.x), gated(g.y, u.y), gated(g.z, u.z), gated(g.w, u.w));
}

// q, k and v of a decoder layer straight from the partial sums of their projections (up to three sets of
// partials: the three matrices of one few-row launch, or K from one split-K launch and Q, V from another),
// with the rotary embedding of q and k: what the plain reductions followed by rope_kernel compute, value for
// value (sum in slice order, rounded to bf16, turned in fp32 at positions[m], rounded), in one launch.
// A thread owns 16 columns: of a q or k head the 8 low channels from 8 j on and the 8 high channels they pair
// with (the angles are computed once per pair, as in rope_kernel); of v 16 consecutive columns.
__global__ __launch_bounds__(256) void qkv_finish_kernel(
    QkvParts P, uint16_t* __restrict__ k, uint16_t* __restrict__ q, uint16_t* __restrict__ v, int Hq, int Hkv,
    int d, const int32_t* __restrict__ positions, float rope_c) {
    const int g16 = d / 16, M = P.parts[0].M;
    const int units = (Hq + 2 * Hkv) * g16;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int m = (int)(id / units);
    if (m >= M) return;
    int unit = (int)(id - (int64_t)m * units);
    int mat = 0;                                         // 0 k, 1 q, 2 v
    if (unit >= Hkv * g16) {
        unit -= Hkv * g16;
        mat = 1;
        if (unit >= Hq * g16) {
            unit -= Hq * g16;
            mat = 2;
        }
    }
    const int head = unit / g16, j = unit - head * g16;
    const int c0 = mat == 2 ? 16 * unit : head * d + 8 * j;
    const int c1 = mat == 2 ? c0 + 8 : c0 + d / 2;
    const SkParts& parts = mat == 0 ? P.parts[0] : (mat == 1 ? P.parts[1] : P.parts[2]);
    const int col0 = mat == 0 ? P.col0[0] : (mat == 1 ? P.col0[1] : P.col0[2]);
    // the angles first (they depend on the position alone): the partial sums' loads are in flight meanwhile
    float sn[8], cs[8];
    if (mat != 2) {
        const float pos = (float)positions[m];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float inv_freq = __builtin_exp2f((float)(8 * j + e) * rope_c);
            sincosf(pos * inv_freq, &sn[e], &cs[e]);
        }
    }
    float a[8], bvals[8];
    sk_sum_tiles2(parts, m, col0 + c0, c1 - c0, a, bvals);
    uint32_t lw[4], hw[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        lw[p] = pack_bf16(a[2 * p], a[2 * p + 1]);
        hw[p] = pack_bf16(bvals[2 * p], bvals[2 * p + 1]);
    }
    const int width = mat == 1 ? Hq * d : Hkv * d;
    uint16_t* dst = (mat == 0 ? k : (mat == 1 ? q : v)) + (int64_t)m * width;
    if (mat != 2) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            float rl[2], rh[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const float lo = e ? bf16_hi(lw[p]) : bf16_lo(lw[p]);
                const float hi = e ? bf16_hi(hw[p]) : bf16_lo(hw[p]);
                rl[e] = lo * cs[2 * p + e] - hi * sn[2 * p + e];
                rh[e] = hi * cs[2 * p + e] + lo * sn[2 * p + e];
            }
            lw[p] = pack_bf16(rl[0], rl[1]);
            hw[p] = pack_bf16(rh[0], rh[1]);
        }
    }
    *reinterpret_cast<uint4*>(dst + c0) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
    *reinterpret_cast<uint4*>(dst + c1) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
}

int launch_qkv_finish(const QkvParts& P, uint16_t* k, uint16_t* q, uint16_t* v, int Hq, int Hkv, int d,
                      const int32_t* positions, float theta, hipStream_t s) {
    const int64_t threads = (int64_t)P.parts[0].M * (Hq + 2 * Hkv) * (d / 16);
    if (threads == 0) return VITCOP_OK;
    hipLaunchKernelGGL(qkv_finish_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, P, k, q, v, Hq,
                       Hkv, d, positions, -2.0f * std::log2(theta) / (float)d);
    return launch_status("qkv_finish");
}

// With this many column groups one workgroup per group already keeps most CUs streaming, at a
// higher rate each, and the partial tiles and their reduction are saved.
constexpr int SK_DIRECT_GROUPS = 128;
static bool skinny_direct(int M, int N, bool want_sumsq) {
    return !want_sumsq && (N + SK_COLS - 1) / SK_COLS >= SK_DIRECT_GROUPS;
}
static int skinny_workgroups(int M, int N, int K) {
    const int groups = (N + SK_COLS - 1) / SK_COLS, total = groups * (K / SK_UNIT);
    return max(groups, min(SK_MAX_WGS, total / 2));
}

bool gemm_skinny_applies(int M, int N, int K) {
    return M >= 1 && M <= SK_MAX_ROWS && K % SK_UNIT == 0 && K >= 2 * SK_UNIT && N % 8 == 0;
}

size_t gemm_skinny_workspace_bytes(int M, int N, int K) {
    if (!gemm_skinny_applies(M, N, K)) return 0;
    return up256((size_t)2 * skinny_workgroups(M, N, K) * M * SK_COLS * 4);
}

template <int MB>
static int launch_skinny_cfg(const uint16_t* x, int64_t x_stride, const SkMats& mats, int64_t w_stride, int M, int N,
                             int K, int wgs, int units_q, int units_r, float* part,
                             const uint16_t* res, int64_t res_stride, hipStream_t s) {
    auto kern = gemm_skinny_kernel<MB>;
    constexpr size_t lds = (size_t)2 * (MB * 32 + SK_COLS) * 128;
    static std::atomic<bool> attr_set{false};   // set once; a second thread repeating the call is harmless
    if (!attr_set.load(std::memory_order_acquire)) {
        int rc = hip_status(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                (int)lds),
                            "hipFuncSetAttribute(gemm_skinny)");
        if (rc) return rc;
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(wgs), dim3(SK_THREADS), lds, s, x, x_stride, mats, w_stride, M, N, K, units_q,
                       units_r, part, res, res_stride);
    return launch_status("gemm_skinny");
}

bool gemm_skinny_fuses_norm(int M, int N, int K) {
    return gemm_skinny_applies(M, N, K) && !skinny_direct(M, N, false) && partial_reduce_fuses_norm(N);
}

// Adds up the partial sums of a launch and finishes the rows: plain (+ residual, + norm side output),
// with the RMSNorm of the finished row (ln_w), or as the gated MLP activation (gated_out; N = 2 F).
int launch_partial_reduce(const SkParts& parts, int N, const SkMats& mats, const uint16_t* res, int64_t res_stride,
                          float* sumsq_parts, const uint16_t* ln_w, float eps, uint16_t* norm_out,
                          int64_t norm_stride, uint16_t* gated_out, hipStream_t s) {
    const int M = parts.M;
    if (gated_out != nullptr) {                  // gate and up side by side
        const int64_t threads = (int64_t)M * (N / 16);
        hipLaunchKernelGGL(gemm_skinny_reduce_silu_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                           parts, N / 2, gated_out, (int64_t)(N / 2));
        return launch_status("gemm_skinny_reduce_silu");
    }
    if (ln_w != nullptr) {
        hipLaunchKernelGGL(gemm_skinny_reduce_norm_kernel, dim3(M), dim3(256), 0, s, parts, N, mats.y[0],
                           mats.y_stride[0], res, res_stride, ln_w, eps, norm_out, norm_stride);
        return launch_status("gemm_skinny_reduce_norm");
    }
    const int chunks = (N + SK_COLS - 1) / SK_COLS * 16;
    const int64_t threads = (int64_t)M * chunks;
    hipLaunchKernelGGL(gemm_skinny_reduce_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, parts, N,
                       mats, res, res_stride, sumsq_parts);
    return launch_status("gemm_skinny_reduce");
}

bool partial_reduce_fuses_norm(int N) { return N % 8 == 0 && N <= 8 * 256 * SK_NORM_CHUNKS; }

// The launch over the matrices of `mats` (N = all their columns) through partial tiles in `ws`
// (gemm_skinny_workspace_bytes).  res and sumsq_parts only with a single matrix.  With ln_w != nullptr
// (only where gemm_skinny_fuses_norm holds, one matrix, no norm side output) norm_out also receives
// RMSNorm(y) * ln_w.
static int launch_skinny_mats(const uint16_t* x, int64_t x_stride, const SkMats& mats, const uint16_t* res,
                              int64_t res_stride, int M, int N, int K, float* sumsq_parts, void* ws, hipStream_t s,
                              const uint16_t* ln_w, float eps, uint16_t* norm_out, int64_t norm_stride,
                              uint16_t* gated_out = nullptr, SkParts* parts_out = nullptr) {
    const bool direct = gated_out == nullptr && skinny_direct(M, N, sumsq_parts != nullptr);
    const int wgs = direct ? (N + SK_COLS - 1) / SK_COLS : skinny_workgroups(M, N, K);
    float* part = direct ? nullptr : static_cast<float*>(ws);
    const int mb = (M + 31) / 32;
    const int total = (N + SK_COLS - 1) / SK_COLS * (K / SK_UNIT), units_q = total / wgs, units_r = total % wgs;
    int rc;
    if (mb <= 2)
        rc = launch_skinny_cfg<2>(x, x_stride, mats, K, M, N, K, wgs, units_q, units_r, part, res, res_stride, s);
    else if (mb <= 4)
        rc = launch_skinny_cfg<4>(x, x_stride, mats, K, M, N, K, wgs, units_q, units_r, part, res, res_stride, s);
    else if (mb <= 6)
        rc = launch_skinny_cfg<6>(x, x_stride, mats, K, M, N, K, wgs, units_q, units_r, part, res, res_stride, s);
    else
        rc = launch_skinny_cfg<8>(x, x_stride, mats, K, M, N, K, wgs, units_q, units_r, part, res, res_stride, s);
    if (parts_out) *parts_out = SkParts{direct ? nullptr : part, units_q, units_r, K / SK_UNIT, M};
    if (rc || direct) return rc;
    const SkParts parts{part, units_q, units_r, K / SK_UNIT, M};
    if (parts_out) return VITCOP_OK;             // the caller finishes the rows itself
    return launch_partial_reduce(parts, N, mats, res, res_stride, sumsq_parts, ln_w, eps, norm_out, norm_stride,
                                 gated_out, s);
}

// y = x W^T (+ res) [M,N] for M <= 256.  With w2: columns [n_split, N) use w2 and go to y2 (n_split a
// multiple of 128); both outputs have row stride y_stride.
int launch_gemm_skinny(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y, int64_t y_stride,
                       const uint16_t* res, int64_t res_stride, int M, int N, int K, float* sumsq_parts,
                       const uint16_t* w2, uint16_t* y2, int n_split, void* ws, hipStream_t s,
                       const uint16_t* ln_w, float eps, uint16_t* norm_out, int64_t norm_stride) {
    SkMats mats{{w, w2 ? w2 : w, w}, {y, w2 ? y2 : y, y}, {y_stride, y_stride, y_stride},
                {w2 ? n_split : N, N, N}};
    return launch_skinny_mats(x, x_stride, mats, res, res_stride, M, N, K, sumsq_parts, ws, s, ln_w, eps, norm_out,
                              norm_stride);
}

// Three projections of the same input in one launch: y[i] = x w[i]^T, [M, n[i]] dense (n[0] and n[1]
// multiples of 128).
int launch_gemm_skinny3(const uint16_t* x, int64_t x_stride, const uint16_t* const w[3], uint16_t* const y[3],
                        const int n[3], int M, int K, void* ws, hipStream_t s, SkParts* parts_out) {
    SkMats mats{{w[0], w[1], w[2]}, {y[0], y[1], y[2]}, {n[0], n[1], n[2]}, {n[0], n[0] + n[1], n[0] + n[1] + n[2]}};
    return launch_skinny_mats(x, x_stride, mats, nullptr, 0, M, n[0] + n[1] + n[2], K, nullptr, ws, s, nullptr, 0.f,
                              nullptr, 0, nullptr, parts_out);
}

// out = silu(x wg^T) * (x wu^T) [M, F] (F a multiple of 128): both projections in one launch, the
// activation in its reduction.
int launch_gemm_skinny_gated(const uint16_t* x, int64_t x_stride, const uint16_t* wg, const uint16_t* wu, int F,
                             uint16_t* out, int M, int K, void* ws, hipStream_t s) {
    SkMats mats{{wg, wu, wu}, {nullptr, nullptr, nullptr}, {0, 0, 0}, {F, 2 * F, 2 * F}};
    return launch_skinny_mats(x, x_stride, mats, nullptr, 0, M, 2 * F, K, nullptr, ws, s, nullptr, 0.f, nullptr, 0,
                              out);
}

}  // namespace vitcop
