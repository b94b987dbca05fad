// Workgroup-wide exact top-k by radix selection, with the lower index winning
// ties and the survivors emitted in ascending index order (Alg. 1 of the paper
// names only TopK; the tie rule and the order are this library's contract).
//
// Keys are 32-bit unsigned with "smaller key = better".  A non-negative float
// orders like its bit pattern, so "k smallest norms" uses the bits as they are
// and "k largest scores" uses their complement.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vitcop {

constexpr int SEL_THREADS = 1024;

struct SelectShared {
    unsigned hist[256];
    unsigned wave_tot[SEL_THREADS / 64];
    unsigned prefix;
    unsigned kk;
};

// keys: n entries in LDS.  Writes out[r] = base + i for the r-th survivor in
// index order.  Must be called by all SEL_THREADS threads of the workgroup.
__device__ inline void block_select_emit(const unsigned* keys, int n, int keep, int32_t* out,
                                         int base, SelectShared& sh) {
    const int tid = threadIdx.x;
    unsigned prefix = 0, mask = 0, kk = (unsigned)keep;
    if (keep > 0) {
        // four 8-bit digits, most significant first: find the key of rank `keep`
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) sh.hist[tid] = 0;
            __syncthreads();
            for (int i0 = 0; i0 < n; i0 += SEL_THREADS) {        // uniform trip count: ballots below
                const int i = i0 + tid;
                const unsigned k = i < n ? keys[i] : 0u;
                const bool live = i < n && (k & mask) == prefix;
                const unsigned dgt = (k >> shift) & 255u;
                // Scores of one sample share their high bits, so in the early passes most lanes
                // of a wavefront hit the same bin: the lanes that agree with the first live lane
                // are counted with one atomic, the others add individually.
                const unsigned long long live_mask = __builtin_amdgcn_ballot_w64(live);
                if (live_mask != 0) {
                    const int leader = __builtin_ctzll(live_mask);
                    const unsigned d0 = __builtin_amdgcn_readlane(dgt, leader);
                    const unsigned long long same = __builtin_amdgcn_ballot_w64(live && dgt == d0);
                    if ((tid & 63) == leader) atomicAdd(&sh.hist[d0], (unsigned)__builtin_popcountll(same));
                    else if (live && dgt != d0) atomicAdd(&sh.hist[dgt], 1u);
                }
            }
            __syncthreads();
            if (tid < 64) {
                unsigned c0 = sh.hist[4 * tid], c1 = sh.hist[4 * tid + 1];
                unsigned c2 = sh.hist[4 * tid + 2], c3 = sh.hist[4 * tid + 3];
                unsigned s = c0 + c1 + c2 + c3, incl = s;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    unsigned t = __shfl_up(incl, o, 64);
                    if (tid >= o) incl += t;
                }
                unsigned excl = incl - s;
                if (kk > excl && kk <= incl) {
                    unsigned r = kk - excl;
                    unsigned dgt = 0;
                    if (r > c0) { r -= c0; dgt = 1;
                        if (r > c1) { r -= c1; dgt = 2;
                            if (r > c2) { r -= c2; dgt = 3; } } }
                    sh.prefix = prefix | ((4u * tid + dgt) << shift);
                    sh.kk = r;
                }
            }
            __syncthreads();
            prefix = sh.prefix;
            kk = sh.kk;
            mask |= 255u << shift;
        }
    }
    // prefix is now the key of the last survivor; kk of the keys equal to it survive
    const unsigned theta = prefix;
    const unsigned need = keep > 0 ? kk : 0u;

    const int ipt = (n + SEL_THREADS - 1) / SEL_THREADS;
    const int lo = min(n, tid * ipt), hi = min(n, lo + ipt);
    unsigned less = 0, eq = 0;
    for (int i = lo; i < hi; ++i) {
        unsigned k = keys[i];
        less += k < theta;
        eq += k == theta;
    }
    // exclusive scan of (less, eq) packed in 16+16 bits (n <= 16384)
    unsigned packed = less | (eq << 16), incl = packed;
    const int lane = tid & 63, wv = tid >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        unsigned t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    if (lane == 63) sh.wave_tot[wv] = incl;
    __syncthreads();
    unsigned woff = 0;
    for (int w = 0; w < wv; ++w) woff += sh.wave_tot[w];
    unsigned excl = incl - packed + woff;
    unsigned lb = excl & 0xFFFFu, eb = excl >> 16;
    for (int i = lo; i < hi; ++i) {
        unsigned k = keys[i];
        if (k < theta) {
            out[lb + min(eb, need)] = base + i;
            ++lb;
        } else if (k == theta) {
            if (eb < need) out[lb + eb] = base + i;
            ++eb;
        }
    }
}

}  // namespace vitcop
