// Causal prefill attention over the surviving tokens: exact
// softmax(scale Q K^T + causal) V with an online softmax, i.e. what a
// FlashAttention kernel computes (Sec. 1 and Sec. 2.2 rely on that
// compatibility; this is the 4 N^2 d term of Eq. 7).  Head dimension 128.
//
// Layout of the computation (wave64, v_mfma_f32_32x32x16_bf16):
//  * a workgroup of 4 wavefronts owns 128 consecutive queries of one
//    (sample, head); each wavefront owns 32 of them;
//  * keys/values stream through LDS in tiles of 64 keys;
//  * scores are computed TRANSPOSED, S^T = K Q^T, so that every lane holds
//    scores of a single query (its column): the running max / sum are
//    per-lane scalars plus one exchange with lane^32, and the probabilities
//    are already laid out as the B operand of the second product
//    O^T += V^T P^T — they never leave registers;
//  * V is written to LDS transposed (channel-major) with the keys of each
//    group of 32 permuted so that the 8 keys a lane needs are contiguous.
#include <atomic>
#include <type_traits>

#include "vitcop_internal.h"
#include "device_utils.h"
#include <algorithm>

namespace vitcop {

constexpr int AT_D = 128;
constexpr int AT_BM = 128;
constexpr int AT_BN = 64;
constexpr int AT_THREADS = 256;
constexpr int AT_VLD = AT_BN + 8;    // bf16 per V^T row in LDS (144 B)

template <int D>
__global__ __launch_bounds__(AT_THREADS) void attn_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, uint16_t* __restrict__ out, float* __restrict__ lse,
    int N, int Hq, int Hkv, float scale_log2e, int causal) {
    static_assert(D == 64 || D == 128, "head dimension");
    constexpr int KLD = D + 8;            // bf16 per K row in LDS (odd multiple of 16 B: conflict-free reads)
    constexpr int DC = D / 16;            // 16-channel MFMA steps of Q K^T
    constexpr int DB = D / 32;            // 32-channel blocks of the output
    constexpr int KCH = D / 8;            // 16-byte chunks per K/V row
    constexpr int KLOADS = AT_BN * KCH / AT_THREADS;   // K chunks per thread per tile (4 or 2)
    __shared__ __attribute__((aligned(16))) uint16_t Ks[AT_BN * KLD];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[D * AT_VLD];

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    // Late query blocks carry the most keys under the causal mask.  The query block is the
    // slowest grid index and is reversed, so workgroups start in order of decreasing work over
    // all heads and samples (longest first keeps the CUs evenly loaded to the end).
    const int qb = causal ? (int)gridDim.z - 1 - (int)blockIdx.z : (int)blockIdx.z;
    const int h = blockIdx.x, b = blockIdx.y;
    const int hk = h / (Hq / Hkv);
    const int q0 = qb * AT_BM, wq0 = q0 + 32 * wv;
    const int64_t q_rs = (int64_t)Hq * D, kv_rs = (int64_t)Hkv * D;
    const int query = wq0 + l32;

    // Q^T fragments (B operand): lane holds 8 channels of its query per 16-channel step
    bf16x8 qf[DC];
    {
        const uint16_t* qp = q + ((int64_t)b * N + min(query, N - 1)) * q_rs + h * D + 8 * g;
#pragma unroll
        for (int dc = 0; dc < DC; ++dc) qf[dc] = *reinterpret_cast<const bf16x8*>(qp + 16 * dc);
    }

    f32x16 o[DB];
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int kend = causal ? min(N, q0 + AT_BM) : N;
    const int ntiles = (kend + AT_BN - 1) / AT_BN;
    const int wave_kend = causal ? min(N, wq0 + 32) : N;
    const uint16_t* kbase = k + (int64_t)b * N * kv_rs + hk * D;
    const uint16_t* vbase = v + (int64_t)b * N * kv_rs + hk * D;

    const int vkq = tid & 15, vc = tid >> 4;      // V: key quad, channel chunk (threads with vc >= KCH idle)
    const bool v_active = vc < KCH;
    // position of the key quad inside its row of V^T: swap the two low bits of the quad index
    const int vpq = (vkq & ~3) | ((vkq & 1) << 1) | ((vkq >> 1) & 1);
    u32x4 kr[KLOADS], vr[4];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int j = 0; j < KLOADS; ++j) {
            const int id = tid + AT_THREADS * j;
            const int key = min(t * AT_BN + id / KCH, N - 1);
            kr[j] = *reinterpret_cast<const u32x4*>(kbase + key * kv_rs + (id % KCH) * 8);
        }
        if (v_active) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int key = min(t * AT_BN + 4 * vkq + j, N - 1);
                vr[j] = *reinterpret_cast<const u32x4*>(vbase + key * kv_rs + vc * 8);
            }
        }
    };
    load_tile(0);

    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < KLOADS; ++j) {
            const int id = tid + AT_THREADS * j;
            *reinterpret_cast<u32x4*>(&Ks[(id / KCH) * KLD + (id % KCH) * 8]) = kr[j];
        }
        if (v_active) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t w0 = vr[0][p], w1 = vr[1][p], w2 = vr[2][p], w3 = vr[3][p];
                uint2 ev, od;
                ev.x = (w0 & 0xFFFFu) | (w1 << 16);
                ev.y = (w2 & 0xFFFFu) | (w3 << 16);
                od.x = (w0 >> 16) | (w1 & 0xFFFF0000u);
                od.y = (w2 >> 16) | (w3 & 0xFFFF0000u);
                *reinterpret_cast<uint2*>(&Vt[(vc * 8 + 2 * p) * AT_VLD + vpq * 4]) = ev;
                *reinterpret_cast<uint2*>(&Vt[(vc * 8 + 2 * p + 1) * AT_VLD + vpq * 4]) = od;
            }
        }
        __syncthreads();
        if (t + 1 < ntiles) load_tile(t + 1);
        if (t * AT_BN >= wave_kend) continue;     // every key of this tile is masked for this wave

        // S^T = K Q^T for the two 32-key halves of the tile
        f32x16 s[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
            for (int dc = 0; dc < DC; ++dc) {
                const bf16x8 a = *reinterpret_cast<const bf16x8*>(
                    &Ks[(kt * 32 + l32) * KLD + dc * 16 + g * 8]);
                s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[dc], s[kt], 0, 0, 0);
            }
        }
        // lane holds, for its query, keys  t*64 + kt*32 + 8*(r/4) + 4*g + r%4
        const int kb0 = t * AT_BN;
        const bool need_mask = (kb0 + AT_BN > N) || (causal && kb0 + AT_BN - 1 > wq0);
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float val = s[kt][r] * scale_log2e;
                if (need_mask) {
                    const int key = kb0 + kt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (key >= N || (causal && key > query)) val = -INFINITY;
                }
                s[kt][r] = val;
                mx = fmaxf(mx, val);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);          // finite: key 0 is visible to every query
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        bf16x8 pf[2][2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                float e[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    e[i] = __builtin_amdgcn_exp2f(s[kt][8 * tt + i] - m_new);
                    psum += e[i];
                }
                uint4 pk;
                pk.x = pack_bf16(e[0], e[1]);
                pk.y = pack_bf16(e[2], e[3]);
                pk.z = pack_bf16(e[4], e[5]);
                pk.w = pack_bf16(e[6], e[7]);
                pf[kt][tt] = __builtin_bit_cast(bf16x8, pk);
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        // O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8*>(
                        &Vt[(db * 32 + l32) * AT_VLD + kt * 32 + tt * 16 + g * 8]);
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[kt][tt], o[db], 0, 0, 0);
                }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (query < N) {
        const float inv = 1.0f / l_tot;
        uint16_t* op = out + ((int64_t)b * N + query) * q_rs + h * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                uint2 pk;
                pk.x = pack_bf16(o[db][4 * r4] * inv, o[db][4 * r4 + 1] * inv);
                pk.y = pack_bf16(o[db][4 * r4 + 2] * inv, o[db][4 * r4 + 3] * inv);
                *reinterpret_cast<uint2*>(op + db * 32 + 8 * r4 + 4 * g) = pk;
            }
        if (lse && g == 0)
            lse[((int64_t)b * Hq + h) * N + query] =
                (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    }
}

// ---------------------------------------------------------------------------
// The kernel for head dimension 128 (the one above remains for 64, and for K/V spans beyond 32-bit byte
// offsets).  A workgroup of 4 wavefronts owns 128 U queries, each wavefront U blocks of 32: with U = 2 (long
// sequences) every K and V^T fragment read from LDS feeds two MFMAs; with U = 1 (the few hundred tokens that
// survive pruning) a wavefront's chain per key tile is half as long and there are twice the workgroups.
// K and V tiles (64 keys) arrive by direct
// global -> LDS loads into a ring of four stages; both stay row-major in LDS,
// padded per KiB; V^T fragments come from the transposing LDS read
// (ds_read_b64_tr_b16), so nothing is staged in or shuffled through registers.
// The reference of the exponentials is only raised when a score exceeds it by
// more than 2^8 (the accumulators are rescaled then); the normalisation at the
// end makes the result independent of which reference was used.
// ---------------------------------------------------------------------------
constexpr int AW_BM = 256;            // queries per workgroup with two query blocks per wavefront (128 with one)
constexpr int AW_BN = 64;
// LDS layout of a 64-key tile (rows of 256 B): one direct-to-LDS load writes 1 KiB = the four
// rows {i, i+16, i+32, i+48}, so row r sits at (r % 16) * (1024 + pad) + (r / 16) * 256.
// The pad after every KiB shifts consecutive keys across the banks: 16 B for K (16-byte
// fragment reads of 16 consecutive keys), 64 B for V (8-byte transposing reads: 32 lanes = 4 consecutive
// keys x 64 B).  Every fragment address is then one per-lane base + a constant.
constexpr int AW_KGRP = 1024 + 16;
constexpr int AW_VGRP = 1024 + 64;
constexpr int AW_KTILE = 16 * AW_KGRP;           // 16640 B
constexpr int AW_VTILE = 16 * AW_VGRP;           // 16896 B
constexpr int AW_STAGE = AW_KTILE + AW_VTILE;    // K then V
constexpr int AW_STAGES = 4;
constexpr float AW_RESCALE_GAP = 8.0f;

typedef __attribute__((ext_vector_type(4))) short s16x4;

// Transposing LDS read (ds_read_b64_tr_b16): lane 16*h + 4*e + a passes the address of 4
// consecutive 16-bit values; it receives, for j = 0..3, element (lane & 3) of the quadruple
// addressed by lane 16*h + 4*j + ((lane >> 2) & 3).
__device__ __forceinline__ s16x4 lds_read_tr16(unsigned addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)addr);
}

// K and V reach LDS by buffer loads with the LDS modifier (16 bytes per lane, global -> LDS without passing
// through registers: lane L's data lands at M0 + 16*L).  They are written as inline assembly on purpose: for
// the builtins the compiler makes every later LDS read wait for ALL such loads in flight, which would undo
// the prefetch; completion is tracked by explicit vmcnt waits before the barrier that publishes a tile.

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// Vector work of the softmax of one 32-key stage (all query blocks of the wavefront), as a list of single
// instructions in issue order.  The pipeline block below cuts the list into as many runs as it has MFMAs
// (16 per query block) and puts one run behind each, with scheduling barriers in between, so that the
// matrix pipe and the vector pipe stay busy together; the order keeps every instruction a
// few issue slots away from the producer of its operands.
//   kinds: MASK (diagonal and ragged tiles only) score := -inf where the key is not visible;
//   MAX5 five 3-input maxima of the lane's 16 scores; MAX3 their reduction to one; FMA argument of
//   an exponential, score * scale - reference; EXP; ADD2 sum of two neighbours, added to one of
//   two running partial sums (few values stay live); CVT pack two probabilities to bf16; TREE the
//   two partial sums combined, then the update of the running denominator.
//   (A dot-product instruction with (1, 1) would sum a packed pair in one go, but it was measured
//   slower: it does not run beside the MFMAs the way plain vector instructions do.)
// The list has two parts.  Part 1 (masks and maxima) fills the first `check` runs; after them the
// block compares each lane's maximum with a threshold and, rarely, raises references (see there).
// Part 2 (everything that needs the reference) fills the remaining runs.
enum SmKind : int { SM_MASK, SM_MAX5, SM_MAX3, SM_FMA, SM_EXP, SM_ADD2, SM_CVT, SM_TREE };
struct SmOp {
    int kind, u, i;
};
constexpr int SM_NOPS = 2 * 16 + 2 * (5 + 3) + 2 * (16 + 16 + 8 + 8 + 2);      // for two query blocks
struct SmTable {
    SmOp op[SM_NOPS];
    int start[33];       // run r is op[start[r]] .. op[start[r+1]-1]
    int check;           // the reference check sits between run check-1 and run check
    int slots;           // runs = MFMAs of a pipeline block: 16 per query block
};
// U query blocks per wavefront (1 or 2)
constexpr SmTable make_sm_table(bool masked, int U) {
    SmTable t{};
    int n = 0;
    const int slots = 16 * U;
    t.slots = slots;
    if (masked)
        for (int i = 0; i < 16; ++i)
            for (int u = 0; u < U; ++u) t.op[n++] = {SM_MASK, u, i};
    // part 1, the query blocks interleaved
    for (int u = 0; u < U; ++u)
        for (int i = 0; i < 5; ++i) t.op[n++] = {SM_MAX5, u, i};
    for (int i = 0; i < 3; ++i)
        for (int u = 0; u < U; ++u) t.op[n++] = {SM_MAX3, u, i};
    const int n1 = n;
    // part 2 in groups of four scores (group g: query block g / 4, scores 4 (g % 4) ..+3),
    // software pipelined: arguments of group ph, exponentials of group ph-1, sums and packing
    // of group ph-2; the tree of a query block follows two phases after its last pair sums
    for (int ph = 0; ph < 4 * U + 5; ++ph) {
        if (ph < 4 * U)
            for (int i = 0; i < 4; ++i) t.op[n++] = {SM_FMA, ph / 4, 4 * (ph % 4) + i};
        if (ph >= 1 && ph < 4 * U + 1)
            for (int i = 0; i < 4; ++i) t.op[n++] = {SM_EXP, (ph - 1) / 4, 4 * ((ph - 1) % 4) + i};
        if (ph >= 2 && ph < 4 * U + 2) {
            const int g = ph - 2;
            for (int i = 0; i < 2; ++i) t.op[n++] = {SM_ADD2, g / 4, 2 * (g % 4) + i};
            for (int i = 0; i < 2; ++i) t.op[n++] = {SM_CVT, g / 4, 2 * (g % 4) + i};
        }
        if (ph >= 7 && (ph - 7) % 4 == 0 && (ph - 7) / 4 < U)       // query block u: pair sums done in phase 4u + 5
            for (int i = 0; i < 2; ++i) t.op[n++] = {SM_TREE, (ph - 7) / 4, i};
    }
    // split into `slots` runs of about equal issue time (a mask is a compare and a select, an
    // exponential takes twice as long as a plain instruction, a pair sum from the third on is two
    // adds); part 1 gets whole runs
    auto weight = [](const SmOp& o) {
        return (o.kind == SM_MASK || o.kind == SM_EXP || (o.kind == SM_ADD2 && o.i >= 2)) ? 2 : 1;
    };
    int w1 = 0, w2 = 0;
    for (int k = 0; k < n1; ++k) w1 += weight(t.op[k]);
    for (int k = n1; k < n; ++k) w2 += weight(t.op[k]);
    const int w_check = 6;       // compare, branch and the registers the rare path sets up
    int runs1 = ((w1 + w_check) * slots + (w1 + w_check + w2) / 2) / (w1 + w_check + w2);
    if (runs1 < 1) runs1 = 1;
    t.check = runs1;
    int acc = 0, r = 0;
    t.start[0] = 0;
    for (int k = 0; k < n1; ++k) {
        acc += weight(t.op[k]);
        while (r < runs1 - 1 && acc * runs1 >= w1 * (r + 1)) t.start[++r] = k + 1;
    }
    while (r < runs1) t.start[++r] = n1;
    acc = 0;
    const int runs2 = slots - runs1;
    for (int k = n1; k < n; ++k) {
        acc += weight(t.op[k]);
        while (r < slots - 1 && acc * runs2 >= w2 * (r - runs1 + 1)) t.start[++r] = k + 1;
    }
    while (r < slots) t.start[++r] = n;
    return t;
}
template <int U, bool MASKED>
constexpr SmTable SM_TABLE_OF = make_sm_table(MASKED, U);

template <bool CAUSAL, int U>
__global__ __launch_bounds__(256) void attn_wide_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
    const uint16_t* __restrict__ v, uint16_t* __restrict__ out, float* __restrict__ lse,
    int N, int Hq, int Hkv, float scale_log2e, int n_qb, int n_heads, int group) {
    extern __shared__ __attribute__((aligned(1024))) char aw_lds[];
    static_assert(U == 1 || U == 2, "query blocks per wavefront");
    constexpr int BM = 128 * U, QW = 32 * U;       // queries per workgroup and per wavefront

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, g = lane >> 5;
    // Workgroup -> (sample*head, query block).  The (sample, head) pairs are taken in groups of
    // `group`; inside a group the query blocks go from the last (most keys under the causal
    // mask) to the first, all heads of the group for each.  So at any time the chip works on
    // few heads and many of their query blocks, which stream the same K and V rows at the
    // same pace and share them in L2, while work still starts in order of decreasing length.
    // Consecutive workgroup ids go to different XCDs (each with its own L2): with a group size
    // that is a multiple of 8 a head keeps its XCD for all its query blocks, and the heads
    // of one XCD are consecutive, i.e. they share their K/V head under grouped-query attention.
    int qb, hb;
    {
        const int id = blockIdx.x;
        const int grp = id / (n_qb * group);
        const int first = grp * group;
        const int gsz = min(group, n_heads - first);
        const int rem = id - first * n_qb;
        const int r = rem / gsz, j = rem - r * gsz;
        hb = first + ((gsz & 7) == 0 ? (j & 7) * (gsz >> 3) + (j >> 3) : j);
        qb = CAUSAL ? n_qb - 1 - r : r;
    }
    const int h = __builtin_amdgcn_readfirstlane(hb % Hq), b = __builtin_amdgcn_readfirstlane(hb / Hq);
    const int hk = __builtin_amdgcn_readfirstlane(h / (Hq / Hkv));
    // Query blocks are aligned to the END of the sequence: a ragged block is then the first one,
    // which has the fewest keys to waste wavefronts on (query indices below 0 do not exist).
    const int q0 = N - (n_qb - qb) * BM, wq0 = q0 + QW * wv;
    const int64_t q_rs = (int64_t)Hq * AT_D, kv_rs = (int64_t)Hkv * AT_D;

    // Q^T fragments of the query blocks
    bf16x8 qf[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int query = max(wq0 + 32 * u + l32, 0);
        const uint16_t* qp = q + ((int64_t)b * N + query) * q_rs + h * AT_D + 8 * g;
#pragma unroll
        for (int dc = 0; dc < 8; ++dc) qf[u][dc] = *reinterpret_cast<const bf16x8*>(qp + 16 * dc);
    }
    // The Q fragments are only ever MFMA operands, which may come from the accumulation
    // registers: keep them there, so the 64 of them do not compete with the accumulators and
    // the softmax for the 256 vector registers (they would be evicted and copied back before
    // every use).
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int dc = 0; dc < 8; ++dc) asm volatile("" : "+a"(qf[u][dc]));

    f32x16 o[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[u][i][r] = 0.f;
    // per query: reference of the exponentials (log2 units), the raw score above which it must be
    // raised, (reference + gap) / scale, and the running denominator
    // (the threshold starts finite so that "maximum - threshold" is never inf - inf)
    float m_ref[U], thr[U], l_run[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        m_ref[u] = -INFINITY;
        thr[u] = -3.0e38f;
        l_run[u] = 0.f;
    }

    const int kend = CAUSAL ? min(N, q0 + BM) : N;
    const int ntiles = (kend + AW_BN - 1) / AW_BN;                 // tiles the workgroup streams
    const int wave_kend = CAUSAL ? wq0 + QW : N;                   // keys this wavefront needs
    const int my_tiles = wq0 + QW > 0 ? (wave_kend + AW_BN - 1) / AW_BN : 0;
    // tiles whose 64 keys are visible to all 64 queries and lie inside the sequence: no masking
    const int full_tiles = min(CAUSAL ? max(wq0, 0) / AW_BN : N / AW_BN, min(N / AW_BN, my_tiles));
    const char* kbase = reinterpret_cast<const char*>(k + (int64_t)b * N * kv_rs + hk * AT_D);
    const char* vbase = reinterpret_cast<const char*>(v + (int64_t)b * N * kv_rs + hk * AT_D);

    // Direct-to-LDS loads.  A tile (64 keys) is 16 KiB groups for K and 16 for V: group g holds rows
    // {g, g+16, g+32, g+48}; a wavefront fetches groups 4*wv .. 4*wv+3 of both, one buffer load of 16 bytes
    // per lane each: lane L carries row g + 16*(L/16), 16-byte chunk L%16.  The address of a load is split so
    // that nothing per-lane ever changes: the descriptor holds the base of this (sample, KV head), the scalar
    // offset the tile and the row group, and ONE vector register the lane's row and chunk.  A load is then
    // three instructions and no vector arithmetic.
    // Rows past the end of the sequence are out of the descriptor's range and arrive as zeros (the scores of
    // those keys are masked, and their zero V rows meet zero probabilities).
    const unsigned lds_base0 = __builtin_amdgcn_readfirstlane(
        (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)aw_lds);
    const unsigned row_bytes = (unsigned)(kv_rs * 2);
    const unsigned tile_stride = AW_BN * row_bytes;
    const unsigned n_rec = (unsigned)(N - 1) * row_bytes + AT_D * 2;      // through the last row of THIS head
    auto make_desc = [&](const char* base) __attribute__((always_inline)) {
        const uint64_t a = reinterpret_cast<uint64_t>(base);
        u32x4 d;                          // raw buffer: base address, no stride, byte range, 32-bit data format
        d.x = __builtin_amdgcn_readfirstlane((unsigned)a);
        d.y = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32) & 0xFFFFu);
        d.z = n_rec;
        d.w = 0x00020000u;
        return d;
    };
    const u32x4 k_desc = make_desc(kbase), v_desc = make_desc(vbase);
    const unsigned lane_off = (unsigned)(4 * wv + 16 * (lane >> 4)) * row_bytes + ((unsigned)(lane & 15) << 4);
    // load j of tile t: row group 4*wv + j/2 of K (j even) or V (j odd)
    auto issue_one = [&](int t, int j) __attribute__((always_inline)) {
        const int i = j >> 1;
        const unsigned stage = lds_base0 + (t % AW_STAGES) * AW_STAGE;
        const unsigned dst = (j & 1) ? stage + AW_KTILE + (4 * wv + i) * AW_VGRP : stage + (4 * wv + i) * AW_KGRP;
        const unsigned off = (unsigned)t * tile_stride + (unsigned)i * row_bytes;
        if (j & 1)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                         :: "s"(dst), "v"(lane_off), "s"(v_desc), "s"(off) : "memory");
        else
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                         :: "s"(dst), "v"(lane_off), "s"(k_desc), "s"(off) : "memory");
    };
    auto issue_tile = [&](int t) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 8; ++j) issue_one(t, j);
    };

    // Software pipeline over "stages" of 32 keys (two per tile).  For stage c, with all U query
    // blocks: S(c) = 8 U MFMAs, softmax(c) = vector work, PV(c) = 8 U MFMAs.  One straight-line
    // block per stage holds softmax(c) next to the MFMAs of PV(c-1) and S(c+1), which do not
    // depend on it; the two MFMA streams are interleaved so that no accumulator is touched
    // twice in a row.  Score accumulators and probability fragments are double buffered by
    // stage parity.
    f32x16 s[2][U];                  // [parity][query block]
    bf16x8 pf[2][U][2];              // [parity][query block][16-key half]

    // lane roles for the transposing V^T read: lane = 16*h16 + 4*e + a supplies the address of
    // key (.. + e), channels 16*(h16&1) + 4*a .. +3; it receives channel (lane & 31), 4 keys
    const int tr_e = (lane >> 2) & 3, tr_a = lane & 3, tr_h = lane >> 4;
    // per-lane parts of the fragment addresses (the rest are compile-time constants)
    //   K row kt*32 + l32, bytes 32*dc + 16*g           V row kt*32 + 16*tt + 8*u + 4*g + e,
    //                                                     channels db*32 + 16*(h16&1) + 4*a
    // (kept as 32-bit LDS byte addresses so that the constants fold into the instruction offsets)
    typedef __attribute__((address_space(3))) char lds_char;
    const unsigned lds0 = (unsigned)(uintptr_t)(lds_char*)aw_lds;
    const unsigned k_lane = lds0 + (l32 & 15) * AW_KGRP + (l32 >> 4) * 256 + g * 16;
    const unsigned v_lane = lds0 + AW_KTILE + (4 * g + tr_e) * AW_VGRP + (16 * (tr_h & 1) + 4 * tr_a) * 2;

    // MFMA fragments are read from LDS one pipeline block ahead of their use, into two register
    // sets that alternate with the stage parity (the spare accumulation registers hold them),
    // so no block waits for LDS.
    bf16x8 kfr[2][8];                // K rows of the stage whose scores the block forms
    s16x4 vlo[2][8], vhi[2][8];      // V^T of the stage whose probabilities the block multiplies
    auto load_k_frags = [&](int set, int t, int kt) __attribute__((always_inline)) {
        unsigned Ks = k_lane + (t % AW_STAGES) * AW_STAGE + kt * 512;
        asm("" : "+v"(Ks));          // keep base + constant addressing
#pragma unroll
        for (int dc = 0; dc < 8; ++dc)
            kfr[set][dc] = *(const __attribute__((address_space(3))) bf16x8*)(uintptr_t)(Ks + dc * 32);
    };

    auto scores_only = [&](int par, int t, int kt) __attribute__((always_inline)) {   // prologue: S of the first stage
        const unsigned Ks = k_lane + (t % AW_STAGES) * AW_STAGE + kt * 512;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[par][u][r] = 0.f;
#pragma unroll
        for (int dc = 0; dc < 8; ++dc) {
            const bf16x8 a = *(const __attribute__((address_space(3))) bf16x8*)(uintptr_t)(Ks + dc * 32);
#pragma unroll
            for (int u = 0; u < U; ++u)
                s[par][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[u][dc], s[par][u], 0, 0, 0);
        }
    };
    auto values_only = [&](int par, int set) __attribute__((always_inline)) {   // drain: PV of the last stage
        static_for<0, 8>([&](auto n) {
            constexpr int tt = n.value >> 2, db = n.value & 3;
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            const s16x8 both = __builtin_shufflevector(vlo[set][n.value], vhi[set][n.value], 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8 a = __builtin_bit_cast(bf16x8, both);
#pragma unroll
            for (int u = 0; u < U; ++u)
                o[u][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[par][u][tt], o[u][db], 0, 0, 0);
        });
    };

    // One pipeline block, stage c = 2t + par: softmax of stage c (scores in s[par]) -> pf[par];
    // PV(c-1) with pf[par^1] and S(c+1) -> s[par^1], both from fragment set `par`, which the
    // previous block requested; this block requests set par^1 for the next one: the K rows of
    // stage c+2 = (tile t+1, half par) and the V rows of stage c = (tile t, half par).
    auto stage_block = [&](int par, int t, auto masked_c, bool has_prev) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_c)::value;
        constexpr int SLOTS = 16 * U;
        const int key0 = t * AW_BN + 32 * par;
        // The fragments requested a whole block ago have long arrived; saying so here (a wait on
        // the LDS counter alone) spares the block partial waits: with its own 24 requests queued
        // behind them the 4-bit counter could not express "only the older ones".
        __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0), other counters untouched
        unsigned Ks = k_lane + ((t + 1) % AW_STAGES) * AW_STAGE + par * 512;
        unsigned Vs = v_lane + (t % AW_STAGES) * AW_STAGE + par * 512;
        asm("" : "+v"(Ks));          // keep base + constant addressing
        asm("" : "+v"(Vs));
        // diagonal and ragged tiles: key key0 + 4g + 8(r/4) + r%4 of register r is visible to
        // the lane's query iff it is <= min(query, N-1), i.e. iff 8(r/4) + r%4 <= lim
        int lim[U] = {};
        if constexpr (MASKED) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int query = max(wq0 + 32 * u + l32, 0);      // rows below 0 are never stored
                lim[u] = (CAUSAL ? min(query, N - 1) : N - 1) - key0 - 4 * g;
            }
        }
        // state of the vector work (see SmKind)
        float m5[U][5], m3[U][3], alpha[U];
#pragma unroll
        for (int u = 0; u < U; ++u) alpha[u] = 1.f;
        float e[U][16], ps[U][2];
        uint32_t pk[U][8];
        bool moved = false;          // wave-uniform: some query of this wavefront raised its reference
        auto vector_op = [&](auto kc, auto uc, auto ic) __attribute__((always_inline)) {
            constexpr int kind = kc.value, u = uc.value, i = ic.value;
            const f32x16& sv = s[par][u];
            if constexpr (kind == SM_MASK) {
                if (8 * (i >> 2) + (i & 3) > lim[u]) s[par][u][i] = -INFINITY;
            } else if constexpr (kind == SM_MAX5) {
                // (the empty asm pins the instruction to its run: nothing else needs the maxima before
                // the check, so the compiler would otherwise gather them all right in front of it)
                m5[u][i] = fmaxf(fmaxf(sv[3 * i], sv[3 * i + 1]), sv[3 * i + 2]);
                asm volatile("" : "+v"(m5[u][i]));
            } else if constexpr (kind == SM_MAX3) {
                if constexpr (i == 0) m3[u][0] = fmaxf(fmaxf(m5[u][0], m5[u][1]), m5[u][2]);
                if constexpr (i == 1) m3[u][1] = fmaxf(fmaxf(m5[u][3], m5[u][4]), sv[15]);
                if constexpr (i == 2) m3[u][2] = fmaxf(m3[u][0], m3[u][1]) - thr[u];   // excess over the threshold
                asm volatile("" : "+v"(m3[u][i]));
            } else if constexpr (kind == SM_FMA) {
                e[u][i] = fmaf(sv[i], scale_log2e, -m_ref[u]);
            } else if constexpr (kind == SM_EXP) {
                e[u][i] = __builtin_amdgcn_exp2f(e[u][i]);
            } else if constexpr (kind == SM_ADD2) {
                const float pair = e[u][2 * i] + e[u][2 * i + 1];
                if constexpr (i < 2) ps[u][i] = pair;
                else ps[u][i & 1] += pair;
            } else if constexpr (kind == SM_CVT) {
                pk[u][i] = pack_bf16(e[u][2 * i], e[u][2 * i + 1]);
            } else {
                if constexpr (i == 0) ps[u][0] += ps[u][1];
                if constexpr (i == 1) l_run[u] = fmaf(l_run[u], alpha[u], ps[u][0]);
            }
        };
        // The reference of a query moves only when its scores exceed it by more than the gap, which is
        // rare (and always the case in a wavefront's first stage): the common path only compares the
        // lane's own maximum with the threshold.  When any lane is over, the whole wavefront takes the
        // long way: maxima exchanged between the two wavefront halves (they hold different keys of the
        // same query, so both decide alike), new reference, alpha = exp2(old - new) (exp2(-inf) = 0 at
        // the start) for the rescaling at the end of the block, new threshold.
        auto check_reference = [&]() __attribute__((always_inline)) {
            float excess = m3[0][2];
#pragma unroll
            for (int u = 1; u < U; ++u) excess = fmaxf(excess, m3[u][2]);
            if (__builtin_expect(__builtin_amdgcn_ballot_w64(excess > 0.f) != 0, 0)) {
                moved = true;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const float own = fmaxf(m3[u][0], m3[u][1]);
                    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(own), __float_as_uint(own),
                                                                     false, false);
                    const float mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
                    const float top = fmaxf(m_ref[u], mx * scale_log2e);
                    const float ref_new = (top > m_ref[u] + AW_RESCALE_GAP) ? top : m_ref[u];
                    alpha[u] = __builtin_amdgcn_exp2f(m_ref[u] - ref_new);
                    m_ref[u] = ref_new;
                    thr[u] = fmaxf((ref_new + AW_RESCALE_GAP) / scale_log2e, -3.0e38f);
                }
            }
        };
        // S(c+1) accumulators
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[par ^ 1][u][r] = 0.f;
        // 16 U slots: one MFMA (those of S(c+1) first, so that they are complete when the next
        // block reads them, then the 16 of PV(c-1)), one fragment request, one run of vector work
        auto run_slot = [&](auto slot) __attribute__((always_inline)) {
            constexpr int i = slot.value;
            if constexpr (i < 8 * U) {
                constexpr int dc = i / U, u = i % U;
                s[par ^ 1][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[par][dc], qf[u][dc], s[par ^ 1][u], 0, 0, 0);
            } else {
                if (has_prev) {
                    constexpr int n = (i - 8 * U) / U, u = i % U, tt = n >> 2, db = n & 3;
                    typedef __attribute__((ext_vector_type(8))) short s16x8;
                    const s16x8 both = __builtin_shufflevector(vlo[par][n], vhi[par][n], 0, 1, 2, 3, 4, 5, 6, 7);
                    o[u][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both),
                                                                       pf[par ^ 1][u][tt], o[u][db], 0, 0, 0);
                }
            }
            // fragment requests at an even pace, 2 KiB per 2 U slots (a K fragment is 1 KiB per wavefront,
            // a V^T half 512 B): bunched together they saturate LDS for the four wavefronts in lock-step,
            // right when the tile loads issued after the barrier are writing into it
            if constexpr (i % (2 * U) == 0)
                kfr[par ^ 1][i / (2 * U)] =
                    *(const __attribute__((address_space(3))) bf16x8*)(uintptr_t)(Ks + (i / (2 * U)) * 32);
            if constexpr (U == 1 || (i & 1) == 1) {
                constexpr int half = i / U, n = half >> 1, off = (n >> 2) * 256 + (n & 3) * 64;
                if constexpr ((half & 1) == 0) vlo[par ^ 1][n] = lds_read_tr16(Vs + off);              // keys of slots 0..3
                else vhi[par ^ 1][n] = lds_read_tr16(Vs + off + 8 * AW_VGRP);                          // keys of slots 4..7
            }
            static_for<SM_TABLE_OF<U, MASKED>.start[i], SM_TABLE_OF<U, MASKED>.start[i + 1]>([&](auto k) {
                constexpr SmOp op = SM_TABLE_OF<U, MASKED>.op[k.value];
                vector_op(std::integral_constant<int, op.kind>{}, std::integral_constant<int, op.u>{},
                          std::integral_constant<int, op.i>{});
            });
            __builtin_amdgcn_sched_barrier(0);
        };
        static_for<0, SM_TABLE_OF<U, MASKED>.check>(run_slot);
        check_reference();
        __builtin_amdgcn_sched_barrier(0);
        static_for<SM_TABLE_OF<U, MASKED>.check, SLOTS>(run_slot);
        // the probabilities are consumed in the next block; without this pin the compiler sinks
        // their computation past the end of this block, away from the MFMAs it must hide behind
#pragma unroll
        for (int u = 0; u < U; ++u)
            asm volatile("" ::"v"(pk[u][0]), "v"(pk[u][1]), "v"(pk[u][2]), "v"(pk[u][3]), "v"(pk[u][4]), "v"(pk[u][5]),
                         "v"(pk[u][6]), "v"(pk[u][7]), "v"(l_run[u]));
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                u32x4 w;
                w.x = pk[u][4 * tt]; w.y = pk[u][4 * tt + 1]; w.z = pk[u][4 * tt + 2]; w.w = pk[u][4 * tt + 3];
                pf[par][u][tt] = __builtin_bit_cast(bf16x8, w);
            }
        // rare: some query moved its reference.  PV(c-1) above still belongs to the old one and
        // has been issued; PV(c) comes in the next block.
        if (__builtin_expect(moved, 0)) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[u][db][r] *= alpha[u];
        }
    };
    // Start of tile t.  After the wait and the barrier, tile t+1 has landed everywhere (the 8
    // loads of tile t+2 may still be in flight) and tile t-1 is dead everywhere: its last
    // fragments were requested in the previous block and have arrived (lgkmcnt), so the fetch
    // of tile t+3 may overwrite its stage.
    // (The eight loads of a tile go out together right after the barrier.  Inside the pipeline blocks they were
    // measured 7 to 15 % slower, whether spread one by one over the MFMA slots or as one burst per wavefront,
    // each wavefront in a slot of its own.)
    auto tile_sync = [&](int t) __attribute__((always_inline)) {
        if (t + 2 < ntiles) asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (t + 3 < ntiles) issue_tile(t + 3);
    };
    auto tile_body = [&](int t, auto masked_c, bool first) __attribute__((always_inline)) {
        // even stage c = 2t: PV(c-1) = second half of tile t-1, S(c+1) = second half of tile t
        stage_block(0, t, masked_c, !first);
        // odd stage c = 2t+1: PV(c-1) = first half of tile t, S(c+1) = first half of tile t+1
        stage_block(1, t, masked_c, true);
    };

    issue_tile(0);
    if (ntiles > 1) issue_tile(1);
    if (ntiles > 2) issue_tile(2);
    tile_sync(0);                    // also covers the Q fragments, which were requested first

    int t = 1;
    if (my_tiles > 0) {
        scores_only(0, 0, 0);
        load_k_frags(0, 0, 1);                                          // for S(1) in the first block
        t = 0;
        if (full_tiles > 0) {
            tile_body(0, std::false_type{}, true);
            for (t = 1; t < full_tiles; ++t) {
                tile_sync(t);
                tile_body(t, std::false_type{}, false);
            }
        }
        for (; t < my_tiles; ++t) {
            if (t > 0) tile_sync(t);
            tile_body(t, std::true_type{}, t == 0);
        }
        values_only(1, 0);                                              // drain: PV of the last stage
    }
    for (; t < ntiles; ++t) tile_sync(t);                     // keep feeding the other wavefronts
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int query = wq0 + 32 * u + l32;                          // < N by construction
        const float l_tot = l_run[u] + __shfl_xor(l_run[u], 32, 64);
        if (query >= 0) {
            const float inv = 1.0f / l_tot;
            uint16_t* op = out + ((int64_t)b * N + query) * q_rs + h * AT_D;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    uint2 pk;
                    pk.x = pack_bf16(o[u][db][4 * r4] * inv, o[u][db][4 * r4 + 1] * inv);
                    pk.y = pack_bf16(o[u][db][4 * r4 + 2] * inv, o[u][db][4 * r4 + 3] * inv);
                    *reinterpret_cast<uint2*>(op + db * 32 + 8 * r4 + 4 * g) = pk;
                }
            if (lse && g == 0)
                lse[((int64_t)b * Hq + h) * N + query] =
                    (m_ref[u] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
        }
    }
}

constexpr int AW_U2_MIN_N = 512;   // a wavefront takes two query blocks from this length on,
constexpr int AW_U2_MIN_WGS = 256;  // if that still leaves more workgroups than this

template <bool CAUSAL, int U>
static int launch_attn_wide(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out, float* lse,
                            int B, int N, int Hq, int Hkv, float sl2, hipStream_t s) {
    static std::atomic<bool> attr_set{false};   // set once; a second thread repeating the call is harmless
    constexpr int lds = AW_STAGES * AW_STAGE;
    if (!attr_set.load(std::memory_order_acquire)) {
        const int rc = hip_status(hipFuncSetAttribute((const void*)attn_wide_kernel<CAUSAL, U>,
                                                      hipFuncAttributeMaxDynamicSharedMemorySize, lds),
                                  "hipFuncSetAttribute(attn_wide)");
        if (rc) return rc;
        attr_set.store(true, std::memory_order_release);
    }
    constexpr int BM = 128 * U;
    const int n_qb = (N + BM - 1) / BM;
    const long n_heads = (long)Hq * B;
    if (n_heads * n_qb > 0x7fffffffL) return fail(VITCOP_EUNSUPPORTED, "attention: grid too large");
    // (sample, head) pairs in flight together: few, so that their query blocks share K/V
    // in L2, but enough to fill the 256 CUs twice over (measured: 32 from N = 2048 up)
    const int group = std::max(32, (512 / n_qb + 7) / 8 * 8);
    hipLaunchKernelGGL((attn_wide_kernel<CAUSAL, U>), dim3((unsigned)(n_heads * n_qb)), dim3(256), lds, s, q, k, v,
                       out, lse, N, Hq, Hkv, sl2, n_qb, (int)n_heads, group);
    return launch_status("attn_wide");
}

int launch_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                float* lse, int B, int N, int Hq, int Hkv, int d, float scale, int causal,
                hipStream_t s) {
    if (B == 0 || N == 0) return VITCOP_OK;
    if (N > (1 << 22)) return fail(VITCOP_EUNSUPPORTED, "attention: N=%d above 2^22", N);   // grid.z limit
    const float sl2 = scale * 1.4426950408889634f;
    if (d == 64) {
        dim3 grid(Hq, B, (N + AT_BM - 1) / AT_BM);
        hipLaunchKernelGGL(attn_kernel<64>, grid, dim3(AT_THREADS), 0, s, q, k, v, out, lse, N, Hq, Hkv, sl2,
                           causal);
        return launch_status("attn<64>");
    }
    // the wide kernel addresses K and V of one (sample, KV head) with 32-bit byte offsets
    const bool wide_ok = ((int64_t)N + AW_BN) * Hkv * AT_D * 2 < ((int64_t)1 << 32);
    if (wide_ok) {
        // Two query blocks per wavefront halve the LDS reads per MFMA, which is what long sequences need; one
        // block halves the chain of MFMAs a wavefront runs per key tile and doubles the workgroups, which is
        // what the lengths that survive pruning need (a few hundred tokens: one to six key tiles per workgroup,
        // latency and not throughput): below 512 tokens, or while 256-query workgroups would not fill the CUs.
        const long wgs2 = (long)Hq * B * ((N + AW_BM - 1) / AW_BM);
        if (N >= AW_U2_MIN_N && wgs2 > AW_U2_MIN_WGS)
            return causal ? launch_attn_wide<true, 2>(q, k, v, out, lse, B, N, Hq, Hkv, sl2, s)
                          : launch_attn_wide<false, 2>(q, k, v, out, lse, B, N, Hq, Hkv, sl2, s);
        return causal ? launch_attn_wide<true, 1>(q, k, v, out, lse, B, N, Hq, Hkv, sl2, s)
                      : launch_attn_wide<false, 1>(q, k, v, out, lse, B, N, Hq, Hkv, sl2, s);
    }
    dim3 grid(Hq, B, (N + AT_BM - 1) / AT_BM);
    hipLaunchKernelGGL(attn_kernel<128>, grid, dim3(AT_THREADS), 0, s, q, k, v, out, lse, N, Hq, Hkv, sl2,
                       causal);
    return launch_status("attn");
}

}  // namespace vitcop
