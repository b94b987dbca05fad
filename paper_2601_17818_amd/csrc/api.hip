// C ABI of libvitcop: argument validation on the host (before any HIP call),
// then kernel launches on the caller's stream.  See include/vitcop.h for the
// contract of each entry point.
#include <algorithm>
#include <vector>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "vitcop_internal.h"

namespace vitcop {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_status(hipError_t e, const char* what) {
    if (e == hipSuccess) return VITCOP_OK;
    return fail(VITCOP_EHIP, "%s: %s", what, hipGetErrorString(e));
}

int launch_status(const char* kernel_name) { return hip_status(hipGetLastError(), kernel_name); }

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Carver {   // hands out 256-byte aligned pieces of the caller's workspace
    char* base;
    size_t used = 0;
    explicit Carver(void* p) : base(static_cast<char*>(p)) {}
    template <typename T>
    T* take(size_t bytes) {
        T* r = reinterpret_cast<T*>(base + used);
        used += up256(bytes);
        return r;
    }
};

}  // namespace vitcop

using namespace vitcop;

#define REQUIRE(cond, code, ...)                     \
    do {                                             \
        if (!(cond)) return fail(code, __VA_ARGS__); \
    } while (0)

extern "C" {
#pragma GCC visibility push(default)

const char* vitcop_last_error(void) { return g_err; }
int vitcop_version(void) { return 1; }

/* ---------------------------------------------------------------- filter */

size_t vitcop_filter_visual_workspace_bytes(int B, int N, int H, int d) {
    if (B < 0 || N < 0 || H < 0 || d < 0) return 0;
    return up256((size_t)B * H * ((size_t)N + 1) * sizeof(float));
}

// Everything vitcop_filter_visual checks apart from the workspace.
static int check_filter(const uint16_t* q_cls, const uint16_t* k, int B, int N, int H, int d, int keep,
                        float scale, const int32_t* idx_out) {
    REQUIRE(B >= 0 && N >= 1 && H >= 1, VITCOP_EINVAL, "filter_visual: B=%d N=%d H=%d", B, N, H);
    REQUIRE(keep >= 0 && keep <= N, VITCOP_EINVAL, "filter_visual: keep=%d outside [0,%d]", keep, N);
    REQUIRE(d == 64 || d == 128, VITCOP_EUNSUPPORTED, "filter_visual: d=%d (64 or 128)", d);
    REQUIRE(N <= VITCOP_MAX_CANDIDATES, VITCOP_EUNSUPPORTED, "filter_visual: N=%d > %d", N,
            VITCOP_MAX_CANDIDATES);
    REQUIRE(H <= 256 && (long)H * d <= 2048, VITCOP_EUNSUPPORTED, "filter_visual: H*d=%ld > 2048",
            (long)H * d);
    REQUIRE(std::isfinite(scale) && scale >= 0.f, VITCOP_EINVAL, "filter_visual: scale");
    if (B == 0) return VITCOP_OK;
    REQUIRE(q_cls && k && (idx_out || keep == 0), VITCOP_EINVAL, "filter_visual: null pointer");
    REQUIRE(aligned16(q_cls) && aligned16(k), VITCOP_EINVAL, "filter_visual: q_cls/k not 16-byte aligned");
    return VITCOP_OK;
}

int vitcop_filter_visual(const uint16_t* q_cls, const uint16_t* k, int B, int N, int H, int d,
                         int keep, float scale, float* scores_out, int32_t* idx_out, void* ws,
                         size_t ws_bytes, void* stream) {
    int rc = check_filter(q_cls, k, B, N, H, d, keep, scale, idx_out);
    if (rc || B == 0) return rc;
    REQUIRE(ws && ws_bytes >= vitcop_filter_visual_workspace_bytes(B, N, H, d), VITCOP_EWORKSPACE,
            "filter_visual: workspace needs %zu bytes", vitcop_filter_visual_workspace_bytes(B, N, H, d));
    if (scale == 0.f) scale = 1.0f / std::sqrt((float)d);
    return launch_filter(q_cls, k, B, N, H, d, keep, scale, scores_out, idx_out,
                         static_cast<float*>(ws), static_cast<hipStream_t>(stream));
}

int vitcop_filter_visual_static(const uint16_t* q_cls, const uint16_t* k, int B, int N, int H, int d,
                                int keep, float scale, float* scores_out, int32_t* idx_out, void* stream) {
    int rc = check_filter(q_cls, k, B, N, H, d, keep, scale, idx_out);
    if (rc || B == 0) return rc;
    const size_t need = (size_t)B * H * ((size_t)N + 1) * sizeof(float);
    REQUIRE(need <= VITCOP_FILTER_STATIC_MAX_BYTES, VITCOP_EUNSUPPORTED,
            "filter_visual_static: B*H*(N+1)*4 = %zu bytes of logits exceed the built-in scratch of %u bytes "
            "(use vitcop_filter_visual with a workspace)", need, (unsigned)VITCOP_FILTER_STATIC_MAX_BYTES);
    float* logits = nullptr;
    rc = filter_static_scratch(&logits);       // no allocation: the address of the library's own array
    if (rc) return rc;
    if (scale == 0.f) scale = 1.0f / std::sqrt((float)d);
    return launch_filter(q_cls, k, B, N, H, d, keep, scale, scores_out, idx_out, logits,
                         static_cast<hipStream_t>(stream));
}

/* --------------------------------------------------------- knorm + select */

size_t vitcop_knorm_select_workspace_bytes(int B, int n_vis) {
    (void)B; (void)n_vis;
    return 0;   // norms are written straight to the caller's `norms`
}

int vitcop_knorm_select(const uint16_t* k, int64_t k_row_stride, int64_t k_batch_stride, int B,
                        int T, int Hkv, int d, int vis_start, int n_vis, int keep, float* norms,
                        int32_t* keep_idx_out, unsigned flags, void* ws, size_t ws_bytes,
                        void* stream) {
    (void)ws; (void)ws_bytes;
    REQUIRE(B >= 0 && T >= 0 && Hkv >= 1 && d >= 1, VITCOP_EINVAL, "knorm_select: B=%d T=%d Hkv=%d d=%d",
            B, T, Hkv, d);
    REQUIRE(vis_start >= 0 && n_vis >= 0 && (long)vis_start + n_vis <= T, VITCOP_EINVAL,
            "knorm_select: visual span [%d,%d) outside [0,%d)", vis_start, vis_start + n_vis, T);
    REQUIRE(keep >= 0 && keep <= n_vis, VITCOP_EINVAL, "knorm_select: keep=%d outside [0,%d]", keep, n_vis);
    REQUIRE((flags & ~(VITCOP_NORMS_PRECOMPUTED | VITCOP_NORMS_SQUARED)) == 0, VITCOP_EINVAL,
            "knorm_select: unknown flags 0x%x", flags);
    REQUIRE(!(flags & VITCOP_NORMS_SQUARED) || (flags & VITCOP_NORMS_PRECOMPUTED), VITCOP_EINVAL,
            "knorm_select: SQUARED needs PRECOMPUTED");
    REQUIRE(n_vis <= VITCOP_MAX_CANDIDATES, VITCOP_EUNSUPPORTED, "knorm_select: n_vis=%d > %d", n_vis,
            VITCOP_MAX_CANDIDATES);
    const long row = (long)Hkv * d;
    const bool pre = flags & VITCOP_NORMS_PRECOMPUTED;
    if (!pre) {
        REQUIRE(row % 8 == 0, VITCOP_EUNSUPPORTED, "knorm_select: Hkv*d=%ld not a multiple of 8", row);
        REQUIRE(k_row_stride >= row && k_row_stride % 8 == 0 && k_batch_stride % 8 == 0 &&
                    k_batch_stride >= 0,
                VITCOP_EINVAL, "knorm_select: strides (%lld, %lld)", (long long)k_row_stride,
                (long long)k_batch_stride);
    }
    if (B == 0 || T == 0) return VITCOP_OK;
    REQUIRE(keep_idx_out, VITCOP_EINVAL, "knorm_select: keep_idx_out is null");
    REQUIRE(norms || n_vis == 0, VITCOP_EINVAL, "knorm_select: norms is null");
    if (!pre) {
        REQUIRE(k && aligned16(k), VITCOP_EINVAL, "knorm_select: k null or not 16-byte aligned");
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!pre) {
        int rc = launch_knorm(k, k_row_stride, k_batch_stride, B, (int)row, vis_start, n_vis, norms, s);
        if (rc) return rc;
    }
    const bool sq = flags & VITCOP_NORMS_SQUARED;
    return launch_select_smallest(norms, 1, 0, n_vis, 0, sq ? 1 : 0, sq ? norms : nullptr, B, T,
                                  vis_start, n_vis, keep, keep_idx_out, s);
}

int vitcop_select_from_sumsq(const float* sumsq_parts, int n_parts, int64_t part_stride, int B,
                             int T, int vis_start, int n_vis, int keep, float* norms_out,
                             int32_t* keep_idx_out, void* stream) {
    REQUIRE(B >= 0 && T >= 0 && n_parts >= 1, VITCOP_EINVAL, "select_from_sumsq: B=%d T=%d parts=%d", B, T,
            n_parts);
    REQUIRE(vis_start >= 0 && n_vis >= 0 && (long)vis_start + n_vis <= T, VITCOP_EINVAL,
            "select_from_sumsq: visual span [%d,%d) outside [0,%d)", vis_start, vis_start + n_vis, T);
    REQUIRE(keep >= 0 && keep <= n_vis, VITCOP_EINVAL, "select_from_sumsq: keep=%d outside [0,%d]", keep,
            n_vis);
    REQUIRE(part_stride >= (int64_t)B * T, VITCOP_EINVAL, "select_from_sumsq: part_stride=%lld < B*T",
            (long long)part_stride);
    REQUIRE(n_vis <= VITCOP_MAX_CANDIDATES, VITCOP_EUNSUPPORTED, "select_from_sumsq: n_vis=%d > %d", n_vis,
            VITCOP_MAX_CANDIDATES);
    if (B == 0 || T == 0) return VITCOP_OK;
    REQUIRE(sumsq_parts && keep_idx_out, VITCOP_EINVAL, "select_from_sumsq: null pointer");
    return launch_select_smallest(sumsq_parts, n_parts, part_stride, T, vis_start, 1, norms_out, B, T,
                                  vis_start, n_vis, keep, keep_idx_out, static_cast<hipStream_t>(stream));
}

/* ---------------------------------------------------------------- compact */

int vitcop_compact(const vitcop_gather_t* tensors, int n_tensors, const int32_t* idx, int B, int T_in,
                   int T_out, void* stream) {
    REQUIRE(n_tensors >= 0 && n_tensors <= VITCOP_MAX_GATHER, VITCOP_EINVAL, "compact: n_tensors=%d", n_tensors);
    REQUIRE(B >= 0 && T_in >= 0 && T_out >= 0, VITCOP_EINVAL, "compact: B=%d T_in=%d T_out=%d", B, T_in, T_out);
    REQUIRE(T_out == 0 || T_in > 0, VITCOP_EINVAL, "compact: T_out=%d rows from an empty source", T_out);
    REQUIRE(n_tensors == 0 || tensors, VITCOP_EINVAL, "compact: tensors is null");
    if (n_tensors == 0 || B == 0 || T_out == 0) return VITCOP_OK;
    REQUIRE(idx, VITCOP_EINVAL, "compact: idx is null");
    for (int i = 0; i < n_tensors; ++i) {
        const vitcop_gather_t& g = tensors[i];
        REQUIRE(g.src && g.dst, VITCOP_EINVAL, "compact: tensor %d has a null pointer", i);
        REQUIRE(g.src != g.dst, VITCOP_EINVAL, "compact: tensor %d is in place", i);
        REQUIRE(g.row_bytes > 0 && g.row_bytes % 4 == 0 && g.src_row_stride_bytes >= g.row_bytes &&
                    g.src_row_stride_bytes % 4 == 0 && g.src_batch_stride_bytes >= 0 &&
                    g.src_batch_stride_bytes % 4 == 0,
                VITCOP_EINVAL, "compact: tensor %d row_bytes/strides (%lld, %lld, %lld)", i,
                (long long)g.row_bytes, (long long)g.src_row_stride_bytes,
                (long long)g.src_batch_stride_bytes);
        REQUIRE((reinterpret_cast<uintptr_t>(g.src) & 3) == 0 && (reinterpret_cast<uintptr_t>(g.dst) & 3) == 0,
                VITCOP_EINVAL, "compact: tensor %d not 4-byte aligned", i);
    }
    return launch_compact(tensors, n_tensors, idx, B, T_out, static_cast<hipStream_t>(stream));
}

/* -------------------------------------------------------------- attention */

size_t vitcop_prefill_attn_workspace_bytes(int B, int N, int Hq, int Hkv, int d) {
    (void)B; (void)N; (void)Hq; (void)Hkv; (void)d;
    return 0;
}

int vitcop_prefill_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                        float* lse_out, int B, int N, int Hq, int Hkv, int d, float scale, int causal,
                        void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    REQUIRE(B >= 0 && N >= 0 && Hq >= 1 && Hkv >= 1, VITCOP_EINVAL, "prefill_attn: B=%d N=%d Hq=%d Hkv=%d", B,
            N, Hq, Hkv);
    REQUIRE(Hq % Hkv == 0, VITCOP_EINVAL, "prefill_attn: Hq=%d not a multiple of Hkv=%d", Hq, Hkv);
    REQUIRE(causal == 0 || causal == 1, VITCOP_EINVAL, "prefill_attn: causal=%d", causal);
    REQUIRE(std::isfinite(scale) && scale >= 0.f, VITCOP_EINVAL, "prefill_attn: scale");
    REQUIRE(d == 64 || d == 128, VITCOP_EUNSUPPORTED, "prefill_attn: d=%d (64 or 128)", d);
    REQUIRE(Hq <= 65535 && B <= 65535, VITCOP_EUNSUPPORTED, "prefill_attn: Hq or B above 65535");
    REQUIRE(N <= (1 << 22), VITCOP_EUNSUPPORTED, "prefill_attn: N=%d above 2^22", N);
    if (B == 0 || N == 0) return VITCOP_OK;
    REQUIRE(q && k && v && out, VITCOP_EINVAL, "prefill_attn: null pointer");
    REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(out), VITCOP_EINVAL,
            "prefill_attn: pointers must be 16-byte aligned");
    if (scale == 0.f) scale = 1.0f / std::sqrt((float)d);
    return launch_attn(q, k, v, out, lse_out, B, N, Hq, Hkv, d, scale, causal, static_cast<hipStream_t>(stream));
}

/* ------------------------------------------------------------- projection */

int vitcop_project_sumsq_parts(int N) { return N > 0 ? gemm_sumsq_parts(N) : 0; }

size_t vitcop_project_workspace_bytes(int M, int N, int K) {
    if (M < 1 || N < 1 || K < 1 || K % 32 != 0 || N % 16 != 0) return 0;
    return gemm_workspace_bytes(M, N, K);
}

int vitcop_project(const uint16_t* x, int64_t x_row_stride, const uint16_t* w, uint16_t* y,
                   int64_t y_row_stride, const uint16_t* residual, int64_t res_row_stride, int M, int N,
                   int K, float* sumsq_parts, void* ws, size_t ws_bytes, void* stream) {
    REQUIRE(M >= 0 && N >= 0 && K >= 1, VITCOP_EINVAL, "project: M=%d N=%d K=%d", M, N, K);
    REQUIRE(K % 32 == 0 && N % 16 == 0, VITCOP_EUNSUPPORTED, "project: K=%d %% 32, N=%d %% 16", K, N);
    REQUIRE(x_row_stride >= K && x_row_stride % 8 == 0 && y_row_stride >= N && y_row_stride % 8 == 0,
            VITCOP_EINVAL, "project: strides (%lld, %lld)", (long long)x_row_stride, (long long)y_row_stride);
    REQUIRE(!residual || (res_row_stride >= N && res_row_stride % 8 == 0), VITCOP_EINVAL,
            "project: residual stride %lld", (long long)res_row_stride);
    REQUIRE((int64_t)M * x_row_stride < ((int64_t)1 << 31) && (int64_t)N * K < ((int64_t)1 << 31),
            VITCOP_EUNSUPPORTED, "project: operand larger than 2^31 elements (4 GiB)");
    if (M == 0 || N == 0) return VITCOP_OK;
    REQUIRE(x && w && y, VITCOP_EINVAL, "project: null pointer");
    REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(residual), VITCOP_EINVAL,
            "project: pointers must be 16-byte aligned");
    REQUIRE(aligned16(ws), VITCOP_EINVAL, "project: workspace must be 16-byte aligned");
    return launch_gemm_ws(x, x_row_stride, w, y, y_row_stride, residual, res_row_stride, M, N, K, sumsq_parts,
                          ws, ws_bytes, static_cast<hipStream_t>(stream));
}

/* ------------------------------------------------------------------ layer */

static int check_layer(const vitcop_layer_t* L) {
    REQUIRE(L, VITCOP_EINVAL, "layer: descriptor is null");
    REQUIRE(L->B >= 1 && L->T >= 1 && L->D >= 32 && L->Hq >= 1 && L->Hkv >= 1, VITCOP_EINVAL,
            "layer: B=%d T=%d D=%d Hq=%d Hkv=%d", L->B, L->T, L->D, L->Hq, L->Hkv);
    REQUIRE(L->Hq % L->Hkv == 0, VITCOP_EINVAL, "layer: Hq=%d not a multiple of Hkv=%d", L->Hq, L->Hkv);
    REQUIRE(L->d == 64 || L->d == 128, VITCOP_EUNSUPPORTED, "layer: d=%d (64 or 128)", L->d);
    REQUIRE(L->D % 32 == 0, VITCOP_EUNSUPPORTED, "layer: D=%d not a multiple of 32", L->D);
    REQUIRE(L->vis_start >= 0 && L->n_vis >= 0 && (long)L->vis_start + L->n_vis <= L->T, VITCOP_EINVAL,
            "layer: visual span [%d,%d) outside [0,%d)", L->vis_start, L->vis_start + L->n_vis, L->T);
    REQUIRE(L->keep >= 0 && L->keep <= L->n_vis, VITCOP_EINVAL, "layer: keep=%d outside [0,%d]", L->keep,
            L->n_vis);
    REQUIRE(L->n_vis <= VITCOP_MAX_CANDIDATES, VITCOP_EUNSUPPORTED, "layer: n_vis=%d > %d", L->n_vis,
            VITCOP_MAX_CANDIDATES);
    REQUIRE(L->T - L->n_vis + L->keep >= 1, VITCOP_EINVAL, "layer: nothing survives");
    return VITCOP_OK;
}

// Scratch of the few-row projection path: the largest need among a layer's projections (rows
// before and after pruning; F = 0: no MLP).
// The need is not monotone in the row count (different paths below 257 and below 1025 rows, slice
// counts that drop as tiles are added), and a schedule sizes its workspace for its longest sequence:
// so a launch of M rows reserves the largest need of any row count up to M.  The need grows with M
// between tile boundaries, which are multiples of 64.
static size_t gemm_scratch_upto(int M, int N, int K) {
    size_t n = gemm_workspace_bytes(M, N, K);
    for (int m = 64; m < M && m <= 1024; m += 64) n = std::max(n, gemm_workspace_bytes(m, N, K));
    return n;
}
static size_t layer_gemm_scratch(int M_all, int M_kept, int D, int qd, int kd, int F, int d = 0) {
    size_t n = gemm_scratch_upto(M_all, kd, D);                                  // K
    n = std::max(n, gemm_scratch_upto(M_kept, qd + kd, D));                      // Q and V
    n = std::max(n, gemm_scratch_upto(M_all, qd + 2 * kd, D));                   // K, Q and V of a layer that keeps all
    if (d > 0) {                                                                 // the same with the rotary embedding
        n = std::max(n, gemm_qkv_workspace_bytes(M_all, qd / d, kd / d, d, D));
        for (int m = 64; m < M_all && m <= 1024; m += 64)
            n = std::max(n, gemm_qkv_workspace_bytes(m, qd / d, kd / d, d, D));
    }
    n = std::max(n, gemm_scratch_upto(M_kept, D, qd));                           // O
    if (F > 0) {
        n = std::max(n, gemm_scratch_upto(M_kept, 2 * F, D));                    // gate and up
        n = std::max(n, gemm_scratch_upto(M_kept, D, F));                        // down
    }
    return n;
}

size_t vitcop_layer_workspace_bytes(const vitcop_layer_t* L) {
    if (check_layer(L) != VITCOP_OK) return 0;
    const size_t B = L->B, T = L->T, Tp = L->T - L->n_vis + L->keep, D = L->D;
    const size_t qd = (size_t)L->Hq * L->d, kd = (size_t)L->Hkv * L->d;
    size_t n = 0;
    n += up256(B * T * kd * 2);                                         // K of every token
    n += up256((size_t)gemm_sumsq_parts((int)kd) * B * T * 4);          // squared-norm partials
    n += up256(B * Tp * 4);                                             // keep list
    n += up256(B * Tp * D * 2);                                         // compacted hidden states
    n += up256(B * Tp * kd * 2);                                        // compacted K
    n += up256(B * Tp * qd * 2);                                        // Q
    n += up256(B * Tp * kd * 2);                                        // V
    n += up256(B * Tp * qd * 2);                                        // attention output
    n += layer_gemm_scratch((int)(B * T), (int)(B * Tp), (int)D, (int)qd, (int)kd, 0);
    return n;
}

int vitcop_layer_prefill(const vitcop_layer_t* L, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_layer(L);
    if (rc) return rc;
    REQUIRE(L->x && L->wq && L->wk && L->wv && L->wo && L->y, VITCOP_EINVAL, "layer: null pointer");
    REQUIRE(aligned16(L->x) && aligned16(L->wq) && aligned16(L->wk) && aligned16(L->wv) &&
                aligned16(L->wo) && aligned16(L->y),
            VITCOP_EINVAL, "layer: pointers must be 16-byte aligned");
    REQUIRE(!L->positions_out || L->positions_in, VITCOP_EINVAL, "layer: positions_out without positions_in");
    REQUIRE(ws && ws_bytes >= vitcop_layer_workspace_bytes(L), VITCOP_EWORKSPACE,
            "layer: workspace needs %zu bytes", vitcop_layer_workspace_bytes(L));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int B = L->B, T = L->T, D = L->D, Tp = L->T - L->n_vis + L->keep;
    const int qd = L->Hq * L->d, kd = L->Hkv * L->d;
    const bool prune = L->keep < L->n_vis;
    const bool want_sel = prune || L->keep_idx || L->norms;
    const int P = gemm_sumsq_parts(kd);

    Carver c(ws);
    uint16_t* k_all = c.take<uint16_t>((size_t)B * T * kd * 2);
    float* parts = c.take<float>((size_t)P * B * T * 4);
    int32_t* idx_ws = c.take<int32_t>((size_t)B * Tp * 4);
    uint16_t* x_kept = c.take<uint16_t>((size_t)B * Tp * D * 2);
    uint16_t* k_kept = c.take<uint16_t>((size_t)B * Tp * kd * 2);
    uint16_t* qb = c.take<uint16_t>((size_t)B * Tp * qd * 2);
    uint16_t* vb = c.take<uint16_t>((size_t)B * Tp * kd * 2);
    uint16_t* ob = c.take<uint16_t>((size_t)B * Tp * qd * 2);
    const size_t gs_bytes = layer_gemm_scratch(B * T, B * Tp, D, qd, kd, 0);
    void* gs = c.take<char>(gs_bytes);
    int32_t* idx = L->keep_idx ? L->keep_idx : idx_ws;

    // K of every token of the layer input, squared norms as a side output
    if (L->ev_kproj_begin) {
        rc = hip_status(hipEventRecord(static_cast<hipEvent_t>(L->ev_kproj_begin), s), "hipEventRecord");
        if (rc) return rc;
    }
    // (nothing to select and nobody asks for the norms: K, Q and V of all tokens go as one launch)
    const bool kqv_together = !want_sel;
    if (kqv_together) {
        const uint16_t* const w3[3] = {L->wk, L->wq, L->wv};
        uint16_t* const y3[3] = {k_all, qb, vb};
        const int n3[3] = {kd, qd, kd};
        rc = launch_gemm_triple_ws(L->x, D, w3, y3, n3, B * T, D, gs, gs_bytes, s);
    } else {
        rc = launch_gemm_ws(L->x, D, L->wk, k_all, kd, nullptr, 0, B * T, kd, D, parts, gs, gs_bytes, s);
    }
    if (rc) return rc;
    if (L->ev_kproj_end) {
        rc = hip_status(hipEventRecord(static_cast<hipEvent_t>(L->ev_kproj_end), s), "hipEventRecord");
        if (rc) return rc;
    }
    if (want_sel) {
        rc = launch_select_smallest(parts, P, (int64_t)B * T, T, L->vis_start, 1, L->norms, B, T,
                                    L->vis_start, L->n_vis, L->keep, idx, s);
        if (rc) return rc;
    }
    const uint16_t* xs = L->x;
    const uint16_t* ks = k_all;
    if (prune) {
        vitcop_gather_t g[3];
        int ng = 0;
        g[ng++] = {L->x, x_kept, (int64_t)D * 2, (int64_t)D * 2, (int64_t)T * D * 2};
        g[ng++] = {k_all, k_kept, (int64_t)kd * 2, (int64_t)kd * 2, (int64_t)T * kd * 2};
        if (L->positions_out) g[ng++] = {L->positions_in, L->positions_out, 4, 4, (int64_t)T * 4};
        rc = launch_compact(g, ng, idx, B, Tp, s);
        if (rc) return rc;
        xs = x_kept;
        ks = k_kept;
    } else if (L->positions_out) {
        rc = hip_status(hipMemcpyAsync(L->positions_out, L->positions_in, (size_t)B * T * 4,
                                       hipMemcpyDeviceToDevice, s),
                        "copy positions");
        if (rc) return rc;
    }
    // Q and V of the survivors only
    if (!kqv_together) {
        rc = launch_gemm_pair_ws(xs, D, L->wq, qb, qd, L->wv, vb, kd, B * Tp, D, gs, gs_bytes, s);
        if (rc) return rc;
    }
    rc = launch_attn(qb, ks, vb, ob, nullptr, B, Tp, L->Hq, L->Hkv, L->d, 1.0f / std::sqrt((float)L->d), 1, s);
    if (rc) return rc;
    return launch_gemm_ws(ob, qd, L->wo, L->y, D, L->residual ? xs : nullptr, D, B * Tp, D, qd, nullptr, gs, gs_bytes, s);
}

/* --------------------------------------------------------------- schedule */

static int check_schedule(const vitcop_schedule_t* S) {
    REQUIRE(S, VITCOP_EINVAL, "schedule: descriptor is null");
    REQUIRE(S->n_layers >= 1 && S->n_stages >= 0, VITCOP_EINVAL, "schedule: n_layers=%d n_stages=%d",
            S->n_layers, S->n_stages);
    REQUIRE(S->n_stages == 0 || (S->prune_layer && S->prune_keep), VITCOP_EINVAL, "schedule: null stage arrays");
    int prev_layer = -1, prev_keep = S->n_vis;
    for (int i = 0; i < S->n_stages; ++i) {
        REQUIRE(S->prune_layer[i] > prev_layer && S->prune_layer[i] < S->n_layers, VITCOP_EINVAL,
                "schedule: stage %d at layer %d (must ascend within [0,%d))", i, S->prune_layer[i],
                S->n_layers);
        REQUIRE(S->prune_keep[i] >= 0 && S->prune_keep[i] <= prev_keep, VITCOP_EINVAL,
                "schedule: stage %d keeps %d of %d", i, S->prune_keep[i], prev_keep);
        prev_layer = S->prune_layer[i];
        prev_keep = S->prune_keep[i];
    }
    vitcop_layer_t L{};
    L.B = S->B; L.T = S->T; L.D = S->D; L.Hq = S->Hq; L.Hkv = S->Hkv; L.d = S->d;
    L.vis_start = S->vis_start; L.n_vis = S->n_vis; L.keep = S->n_vis;
    return check_layer(&L);
}

size_t vitcop_schedule_workspace_bytes(const vitcop_schedule_t* S) {
    if (check_schedule(S) != VITCOP_OK) return 0;
    vitcop_layer_t L{};
    L.B = S->B; L.T = S->T; L.D = S->D; L.Hq = S->Hq; L.Hkv = S->Hkv; L.d = S->d;
    L.vis_start = S->vis_start; L.n_vis = S->n_vis; L.keep = S->n_vis;
    // the largest layer workspace along the schedule (the few-row projection path only needs its
    // scratch once pruning has cut the sequence)
    size_t layer_max = 0;
    int stage = 0;
    for (int l = 0; l < S->n_layers; ++l) {
        L.keep = L.n_vis;
        const bool prune_here = stage < S->n_stages && S->prune_layer[stage] == l;
        if (prune_here) L.keep = S->prune_keep[stage++];
        layer_max = std::max(layer_max, vitcop_layer_workspace_bytes(&L));
        L.T = L.T - L.n_vis + L.keep;
        L.n_vis = L.keep;
    }
    const size_t B = S->B, T = S->T, D = S->D;
    return layer_max + 2 * up256(B * T * D * 2) + 2 * up256(B * T * 4);
}

__global__ void iota_kernel(int32_t* p, int T, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (int32_t)(i % T);
}

int vitcop_schedule_prefill(const vitcop_schedule_t* S, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_schedule(S);
    if (rc) return rc;
    REQUIRE(S->x && S->y_out && S->wq && S->wk && S->wv && S->wo, VITCOP_EINVAL, "schedule: null pointer");
    for (int l = 0; l < S->n_layers; ++l)
        REQUIRE(S->wq[l] && S->wk[l] && S->wv[l] && S->wo[l], VITCOP_EINVAL, "schedule: layer %d has a null weight", l);
    REQUIRE(ws && ws_bytes >= vitcop_schedule_workspace_bytes(S), VITCOP_EWORKSPACE,
            "schedule: workspace needs %zu bytes", vitcop_schedule_workspace_bytes(S));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t B = S->B, T = S->T, D = S->D;
    Carver c(ws);
    uint16_t* hbuf[2] = {c.take<uint16_t>(B * T * D * 2), c.take<uint16_t>(B * T * D * 2)};
    int32_t* pbuf[2] = {c.take<int32_t>(B * T * 4), c.take<int32_t>(B * T * 4)};
    void* lws = c.base + c.used;
    const size_t lws_bytes = ws_bytes - c.used;

    const int64_t npos = (int64_t)B * T;
    hipLaunchKernelGGL(iota_kernel, dim3((unsigned)((npos + 255) / 256)), dim3(256), 0, s, pbuf[0], S->T, npos);
    rc = launch_status("iota");
    if (rc) return rc;

    const uint16_t* h = S->x;
    int cur_T = S->T, cur_vis = S->n_vis, stage = 0, pp = 0;
    for (int l = 0; l < S->n_layers; ++l) {
        vitcop_layer_t L{};
        L.B = S->B; L.T = cur_T; L.D = S->D; L.Hq = S->Hq; L.Hkv = S->Hkv; L.d = S->d;
        L.vis_start = S->vis_start; L.n_vis = cur_vis; L.keep = cur_vis; L.residual = 1;
        L.x = h; L.wq = S->wq[l]; L.wk = S->wk[l]; L.wv = S->wv[l]; L.wo = S->wo[l];
        const bool last = l + 1 == S->n_layers;
        const bool prune_here = stage < S->n_stages && S->prune_layer[stage] == l;
        if (prune_here) {
            L.keep = S->prune_keep[stage++];
            L.positions_in = pbuf[pp];
            L.positions_out = pbuf[pp ^ 1];
        }
        uint16_t* dst = last ? S->y_out : hbuf[l & 1];
        L.y = dst;
        rc = vitcop_layer_prefill(&L, lws, lws_bytes, stream);
        if (rc) return rc;
        if (prune_here) {
            pp ^= 1;
            cur_T = cur_T - cur_vis + L.keep;
            cur_vis = L.keep;
        }
        h = dst;
    }
    if (S->positions_out) {
        rc = hip_status(hipMemcpyAsync(S->positions_out, pbuf[pp], (size_t)B * cur_T * 4,
                                       hipMemcpyDeviceToDevice, s),
                        "copy positions");
    }
    return rc;
}

/* ------------------------------------------------ Visual Information Clustering */

static int check_vic(int B, int n, int D, float d_c, float tau, int n_centers) {
    REQUIRE(B >= 0 && n >= 0 && D >= 8, VITCOP_EINVAL, "vic_cluster: B=%d n=%d D=%d", B, n, D);
    REQUIRE(n <= VITCOP_VIC_MAX_TOKENS, VITCOP_EUNSUPPORTED, "vic_cluster: n=%d above %d", n, VITCOP_VIC_MAX_TOKENS);
    REQUIRE(D % 32 == 0, VITCOP_EUNSUPPORTED, "vic_cluster: D=%d not a multiple of 32", D);
    REQUIRE(B <= 65535, VITCOP_EUNSUPPORTED, "vic_cluster: B above 65535");
    REQUIRE(std::isfinite(d_c) && d_c > 0.f, VITCOP_EINVAL, "vic_cluster: d_c must be positive");
    REQUIRE(std::isfinite(tau) && tau >= 0.f, VITCOP_EINVAL, "vic_cluster: tau must be non-negative");
    REQUIRE(n_centers >= 0 && n_centers <= n, VITCOP_EINVAL, "vic_cluster: n_centers=%d outside [0,%d]", n_centers, n);
    return VITCOP_OK;
}

size_t vitcop_vic_cluster_workspace_bytes(int B, int n, int D) {
    if (B < 0 || n < 0 || n > VITCOP_VIC_MAX_TOKENS || D < 8) return 0;
    return vic_workspace_bytes(B, n);
}

int vitcop_vic_cluster(const uint16_t* feats, int64_t feat_row_stride, int64_t feat_batch_stride,
                       const float* pos, int B, int n, int D, float d_c, float tau, int n_centers,
                       int32_t* labels_out, int32_t* n_clusters_out, float* rho_out, float* delta_out,
                       int32_t* parent_out, float* dist_out, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_vic(B, n, D, d_c, tau, n_centers);
    if (rc) return rc;
    if (B == 0) return VITCOP_OK;
    REQUIRE(n_clusters_out, VITCOP_EINVAL, "vic_cluster: null pointer");
    if (n > 0) {
        REQUIRE(feats && pos && labels_out, VITCOP_EINVAL, "vic_cluster: null pointer");
        REQUIRE(aligned16(feats) && aligned16(pos) && aligned16(dist_out), VITCOP_EINVAL,
                "vic_cluster: feats, pos and dist_out must be 16-byte aligned");
        REQUIRE(feat_row_stride >= D && feat_row_stride % 8 == 0 && feat_batch_stride % 8 == 0 &&
                    (B == 1 || feat_batch_stride >= (int64_t)n * feat_row_stride),
                VITCOP_EINVAL, "vic_cluster: strides");
        REQUIRE((int64_t)n * feat_row_stride < (1LL << 31), VITCOP_EUNSUPPORTED,
                "vic_cluster: one image's features must stay below 2^31 elements");
        const size_t need = vic_workspace_bytes(B, n);
        REQUIRE(ws && ws_bytes >= need, VITCOP_EWORKSPACE, "vic_cluster: workspace %zu < %zu", ws_bytes, need);
        REQUIRE(aligned16(ws), VITCOP_EINVAL, "vic_cluster: workspace must be 16-byte aligned");
    }
    return launch_vic(feats, feat_row_stride, feat_batch_stride, pos, B, n, D, d_c, tau, n_centers, labels_out,
                      n_clusters_out, rho_out, delta_out, parent_out, dist_out, ws, static_cast<hipStream_t>(stream));
}

/* ------------------------------------- collaborative pruning and merging */

size_t vitcop_collab_prune_merge_workspace_bytes(int B, int n) {
    if (B < 0 || n < 0 || n > VITCOP_VIC_MAX_TOKENS) return 0;
    return collab_workspace_bytes(B, n);
}

int vitcop_collab_prune_merge(const uint16_t* feats, int64_t feat_row_stride, int64_t feat_batch_stride,
                              const int32_t* labels, const int32_t* n_clusters, const float* k_norms,
                              int B, int n, int D, int budget, uint16_t* out_feats, int32_t* out_index,
                              int32_t* n_out, int32_t* assign_out, void* ws, size_t ws_bytes, void* stream) {
    REQUIRE(B >= 0 && n >= 0 && D >= 8, VITCOP_EINVAL, "collab_prune_merge: B=%d n=%d D=%d", B, n, D);
    REQUIRE(n <= VITCOP_VIC_MAX_TOKENS, VITCOP_EUNSUPPORTED, "collab_prune_merge: n=%d above %d", n,
            VITCOP_VIC_MAX_TOKENS);
    REQUIRE(D % 8 == 0, VITCOP_EUNSUPPORTED, "collab_prune_merge: D=%d not a multiple of 8", D);
    REQUIRE(budget >= 0, VITCOP_EINVAL, "collab_prune_merge: budget=%d", budget);
    REQUIRE(B <= 65535, VITCOP_EUNSUPPORTED, "collab_prune_merge: B above 65535");
    if (B == 0) return VITCOP_OK;
    REQUIRE(n_clusters && n_out, VITCOP_EINVAL, "collab_prune_merge: null pointer");
    if (n > 0) {
        REQUIRE(feats && labels && k_norms && out_feats && out_index, VITCOP_EINVAL,
                "collab_prune_merge: null pointer");
        REQUIRE(aligned16(feats) && aligned16(out_feats), VITCOP_EINVAL,
                "collab_prune_merge: feats and out_feats must be 16-byte aligned");
        REQUIRE(feat_row_stride >= D && feat_row_stride % 8 == 0 && feat_batch_stride % 8 == 0 &&
                    (B == 1 || feat_batch_stride >= (int64_t)n * feat_row_stride),
                VITCOP_EINVAL, "collab_prune_merge: strides");
    }
    const size_t need = collab_workspace_bytes(B, n);
    REQUIRE(ws && ws_bytes >= need, VITCOP_EWORKSPACE, "collab_prune_merge: workspace %zu < %zu", ws_bytes, need);
    return launch_collab(feats, feat_row_stride, feat_batch_stride, labels, n_clusters, k_norms, B, n, D, budget,
                         out_feats, out_index, n_out, assign_out, ws, static_cast<hipStream_t>(stream));
}

/* ------------------------------------------------------------ decoder layer */

int vitcop_rmsnorm(const uint16_t* x, int64_t x_row_stride, const uint16_t* weight, float eps, uint16_t* y,
                   int64_t y_row_stride, int M, int D, void* stream) {
    REQUIRE(M >= 0 && D >= 8, VITCOP_EINVAL, "rmsnorm: M=%d D=%d", M, D);
    REQUIRE(D % 8 == 0, VITCOP_EUNSUPPORTED, "rmsnorm: D=%d not a multiple of 8", D);
    REQUIRE(std::isfinite(eps) && eps >= 0.f, VITCOP_EINVAL, "rmsnorm: eps");
    if (M == 0) return VITCOP_OK;
    REQUIRE(x && weight && y, VITCOP_EINVAL, "rmsnorm: null pointer");
    REQUIRE(aligned16(x) && aligned16(weight) && aligned16(y), VITCOP_EINVAL, "rmsnorm: pointers must be 16-byte aligned");
    REQUIRE(x_row_stride >= D && x_row_stride % 8 == 0 && y_row_stride >= D && y_row_stride % 8 == 0, VITCOP_EINVAL,
            "rmsnorm: strides");
    return launch_rmsnorm(x, x_row_stride, weight, eps, y, y_row_stride, M, D, static_cast<hipStream_t>(stream));
}

int vitcop_rope(uint16_t* q, uint16_t* k, const int32_t* positions, int B, int N, int Hq, int Hkv, int d,
                float theta, void* stream) {
    REQUIRE(B >= 0 && N >= 0 && Hq >= 0 && Hkv >= 0 && d >= 16, VITCOP_EINVAL, "rope: B=%d N=%d Hq=%d Hkv=%d d=%d", B,
            N, Hq, Hkv, d);
    REQUIRE(d % 16 == 0, VITCOP_EUNSUPPORTED, "rope: d=%d not a multiple of 16", d);
    REQUIRE(std::isfinite(theta) && theta > 1.f, VITCOP_EINVAL, "rope: theta must exceed 1");
    if (B == 0 || N == 0 || (!q && !k)) return VITCOP_OK;
    REQUIRE(positions, VITCOP_EINVAL, "rope: null positions");
    REQUIRE(aligned16(q) && aligned16(k), VITCOP_EINVAL, "rope: pointers must be 16-byte aligned");
    return launch_rope(q, k, positions, (int64_t)B * N, Hq, Hkv, d, theta, static_cast<hipStream_t>(stream));
}

int vitcop_silu_mul(const uint16_t* gate, const uint16_t* up, uint16_t* out, int64_t n_elems, void* stream) {
    REQUIRE(n_elems >= 0 && n_elems % 8 == 0, VITCOP_EINVAL, "silu_mul: n_elems=%ld must be a multiple of 8", (long)n_elems);
    if (n_elems == 0) return VITCOP_OK;
    REQUIRE(gate && up && out, VITCOP_EINVAL, "silu_mul: null pointer");
    REQUIRE(aligned16(gate) && aligned16(up) && aligned16(out), VITCOP_EINVAL, "silu_mul: pointers must be 16-byte aligned");
    return launch_silu_mul(gate, up, out, n_elems, static_cast<hipStream_t>(stream));
}

static int check_decoder_layer(const vitcop_decoder_layer_t* L) {
    REQUIRE(L, VITCOP_EINVAL, "decoder_layer: descriptor is null");
    REQUIRE(L->B >= 1 && L->T >= 1 && L->D >= 32 && L->Hq >= 1 && L->Hkv >= 1 && L->F >= 32, VITCOP_EINVAL,
            "decoder_layer: B=%d T=%d D=%d Hq=%d Hkv=%d F=%d", L->B, L->T, L->D, L->Hq, L->Hkv, L->F);
    REQUIRE(L->Hq % L->Hkv == 0, VITCOP_EINVAL, "decoder_layer: Hq=%d not a multiple of Hkv=%d", L->Hq, L->Hkv);
    REQUIRE(L->d == 64 || L->d == 128, VITCOP_EUNSUPPORTED, "decoder_layer: d=%d (64 or 128)", L->d);
    REQUIRE(L->D % 32 == 0 && L->F % 32 == 0, VITCOP_EUNSUPPORTED, "decoder_layer: D=%d, F=%d must be multiples of 32",
            L->D, L->F);
    REQUIRE(L->vis_start >= 0 && L->n_vis >= 0 && (long)L->vis_start + L->n_vis <= L->T, VITCOP_EINVAL,
            "decoder_layer: visual span [%d,%d) outside [0,%d)", L->vis_start, L->vis_start + L->n_vis, L->T);
    REQUIRE(L->keep >= 0 && L->keep <= L->n_vis, VITCOP_EINVAL, "decoder_layer: keep=%d outside [0,%d]", L->keep,
            L->n_vis);
    REQUIRE(L->n_vis <= VITCOP_MAX_CANDIDATES, VITCOP_EUNSUPPORTED, "decoder_layer: n_vis=%d > %d", L->n_vis,
            VITCOP_MAX_CANDIDATES);
    REQUIRE(L->T - L->n_vis + L->keep >= 1, VITCOP_EINVAL, "decoder_layer: nothing survives");
    REQUIRE(std::isfinite(L->eps) && L->eps >= 0.f && std::isfinite(L->theta) && L->theta > 1.f, VITCOP_EINVAL,
            "decoder_layer: eps or theta");
    REQUIRE((long)L->B * L->T * std::max(L->D, L->F) < (1L << 31), VITCOP_EUNSUPPORTED,
            "decoder_layer: an activation tensor would reach 2^31 elements");
    REQUIRE((L->k_cache == nullptr) == (L->v_cache == nullptr), VITCOP_EINVAL,
            "decoder_layer: k_cache and v_cache go together");
    REQUIRE(!L->k_cache || L->cache_capacity >= L->T - L->n_vis + L->keep, VITCOP_EINVAL,
            "decoder_layer: cache_capacity=%d below the %d kept tokens", L->cache_capacity,
            L->T - L->n_vis + L->keep);
    return VITCOP_OK;
}

size_t vitcop_decoder_layer_workspace_bytes(const vitcop_decoder_layer_t* L) {
    if (check_decoder_layer(L) != VITCOP_OK) return 0;
    const size_t B = L->B, T = L->T, Tp = L->T - L->n_vis + L->keep, D = L->D, F = L->F;
    const size_t qd = (size_t)L->Hq * L->d, kd = (size_t)L->Hkv * L->d;
    size_t n = 0;
    n += up256(B * T * D * 2);                                          // a = RMSNorm(h)
    n += up256(B * T * kd * 2);                                         // K of every token
    n += up256((size_t)gemm_sumsq_parts((int)kd) * B * T * 4);          // squared-norm partials
    n += 2 * up256(B * Tp * 4);                                         // keep list, positions
    n += 2 * up256(B * Tp * D * 2);                                     // gathered h and a
    n += up256(B * Tp * kd * 2);                                        // gathered K
    n += up256(B * Tp * qd * 2) + up256(B * Tp * kd * 2);               // Q, V
    n += up256(B * Tp * qd * 2);                                        // attention output
    n += 2 * up256(B * Tp * D * 2);                                     // h1, b
    n += 3 * up256(B * Tp * F * 2);                                     // gate, up, silu(gate) * up
    n += layer_gemm_scratch((int)(B * T), (int)(B * Tp), (int)D, (int)qd, (int)kd, (int)F, L->d);
    return n;
}

// The layer.  a_pre: RMSNorm(h) * ln1 already computed ([B*T, D] dense), or null.  ln_next / a_next:
// if given, a_next [B*T', D] also receives RMSNorm(y) * ln_next, the next layer's a_pre (fused into
// the down projection's reduction where the few-row path runs it).
static int decoder_layer_run(const vitcop_decoder_layer_t* L, const uint16_t* a_pre, const uint16_t* ln_next,
                             uint16_t* a_next, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_decoder_layer(L);
    if (rc) return rc;
    REQUIRE(L->h && L->positions && L->ln1 && L->ln2 && L->wq && L->wk && L->wv && L->wo && L->wg && L->wu &&
                L->wd && L->y,
            VITCOP_EINVAL, "decoder_layer: null pointer");
    REQUIRE(aligned16(L->h) && aligned16(L->ln1) && aligned16(L->ln2) && aligned16(L->wq) && aligned16(L->wk) &&
                aligned16(L->wv) && aligned16(L->wo) && aligned16(L->wg) && aligned16(L->wu) && aligned16(L->wd) &&
                aligned16(L->y),
            VITCOP_EINVAL, "decoder_layer: pointers must be 16-byte aligned");
    const size_t need = vitcop_decoder_layer_workspace_bytes(L);
    REQUIRE(ws && ws_bytes >= need, VITCOP_EWORKSPACE, "decoder_layer: workspace needs %zu bytes", need);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int B = L->B, T = L->T, D = L->D, F = L->F, Tp = L->T - L->n_vis + L->keep;
    const int qd = L->Hq * L->d, kd = L->Hkv * L->d;
    const bool prune = L->keep < L->n_vis;
    const bool want_sel = prune || L->keep_idx || L->norms;
    const int P = gemm_sumsq_parts(kd);

    Carver c(ws);
    uint16_t* a_all = c.take<uint16_t>((size_t)B * T * D * 2);
    uint16_t* k_all = c.take<uint16_t>((size_t)B * T * kd * 2);
    float* parts = c.take<float>((size_t)P * B * T * 4);
    int32_t* idx_ws = c.take<int32_t>((size_t)B * Tp * 4);
    int32_t* pos_ws = c.take<int32_t>((size_t)B * Tp * 4);
    uint16_t* h_kept = c.take<uint16_t>((size_t)B * Tp * D * 2);
    uint16_t* a_kept = c.take<uint16_t>((size_t)B * Tp * D * 2);
    uint16_t* k_kept = c.take<uint16_t>((size_t)B * Tp * kd * 2);
    uint16_t* qb = c.take<uint16_t>((size_t)B * Tp * qd * 2);
    uint16_t* vb = c.take<uint16_t>((size_t)B * Tp * kd * 2);
    uint16_t* ob = c.take<uint16_t>((size_t)B * Tp * qd * 2);
    uint16_t* h1 = c.take<uint16_t>((size_t)B * Tp * D * 2);
    uint16_t* bb = c.take<uint16_t>((size_t)B * Tp * D * 2);
    uint16_t* gate = c.take<uint16_t>((size_t)B * Tp * F * 2);
    uint16_t* up = c.take<uint16_t>((size_t)B * Tp * F * 2);
    uint16_t* act = c.take<uint16_t>((size_t)B * Tp * F * 2);
    const size_t gs_bytes = layer_gemm_scratch(B * T, B * Tp, D, qd, kd, F, L->d);
    void* gs = c.take<char>(gs_bytes);
    int32_t* idx = L->keep_idx ? L->keep_idx : idx_ws;
    int32_t* pos = L->positions_out ? L->positions_out : pos_ws;

    if (a_pre) {
        a_all = const_cast<uint16_t*>(a_pre);
    } else {
        rc = launch_rmsnorm(L->h, D, L->ln1, L->eps, a_all, D, B * T, D, s);
        if (rc) return rc;
    }
    // K of every token, squared norms (before the rotary embedding) as a side output
    // (nothing to select and nobody asks for the norms: K, Q and V of all tokens go together, and the rotary
    // embedding of q and k with them)
    const bool kqv_together = !want_sel;
    if (kqv_together) {
        rc = launch_gemm_qkv_rope_ws(a_all, D, L->wk, L->wq, L->wv, k_all, qb, vb, L->Hq, L->Hkv, L->d, L->positions,
                                     L->theta, B * T, D, gs, gs_bytes, s);
    } else {
        rc = launch_gemm_ws(a_all, D, L->wk, k_all, kd, nullptr, 0, B * T, kd, D, parts, gs, gs_bytes, s);
    }
    if (rc) return rc;
    if (want_sel) {
        rc = launch_select_smallest(parts, P, (int64_t)B * T, T, L->vis_start, 1, L->norms, B, T, L->vis_start,
                                    L->n_vis, L->keep, idx, s, L->n_vis_samples, L->n_vis_samples_out);
        if (rc) return rc;
    }
    const uint16_t *hs = L->h, *as = a_all;
    uint16_t* ks = k_all;
    const int32_t* ps = L->positions;
    if (prune) {
        vitcop_gather_t g[4] = {{L->h, h_kept, (int64_t)D * 2, (int64_t)D * 2, (int64_t)T * D * 2},
                                {a_all, a_kept, (int64_t)D * 2, (int64_t)D * 2, (int64_t)T * D * 2},
                                {k_all, k_kept, (int64_t)kd * 2, (int64_t)kd * 2, (int64_t)T * kd * 2},
                                {L->positions, pos, 4, 4, (int64_t)T * 4}};
        rc = launch_compact(g, 4, idx, B, Tp, s);
        if (rc) return rc;
        hs = h_kept;
        as = a_kept;
        ks = k_kept;
        ps = pos;
    } else if (L->positions_out) {
        rc = hip_status(hipMemcpyAsync(L->positions_out, L->positions, (size_t)B * T * 4, hipMemcpyDeviceToDevice, s),
                        "copy positions");
        if (rc) return rc;
    }
    if (!kqv_together) {
        rc = launch_gemm_pair_ws(as, D, L->wq, qb, qd, L->wv, vb, kd, B * Tp, D, gs, gs_bytes, s);
        if (rc) return rc;
    }
    if (!kqv_together) {
        rc = launch_rope(qb, ks, ps, (int64_t)B * Tp, L->Hq, L->Hkv, L->d, L->theta, s);
        if (rc) return rc;
    }
    if (L->k_cache && L->v_cache && Tp > 0) {        // the layer's KV cache: rows [0,T') of each sample's block
        const size_t rowb = (size_t)Tp * kd * 2, pitch = (size_t)L->cache_capacity * kd * 2;
        rc = hip_status(hipMemcpy2DAsync(L->k_cache, pitch, ks, rowb, rowb, B, hipMemcpyDeviceToDevice, s),
                        "copy K to the cache");
        if (rc) return rc;
        rc = hip_status(hipMemcpy2DAsync(L->v_cache, pitch, vb, rowb, rowb, B, hipMemcpyDeviceToDevice, s),
                        "copy V to the cache");
        if (rc) return rc;
    }
    rc = launch_attn(qb, ks, vb, ob, nullptr, B, Tp, L->Hq, L->Hkv, L->d, 1.0f / std::sqrt((float)L->d), 1, s);
    if (rc) return rc;
    rc = launch_gemm_norm_ws(ob, qd, L->wo, h1, D, hs, D, B * Tp, D, qd, L->ln2, L->eps, bb, D, gs, gs_bytes, s);
    if (rc) return rc;
    rc = launch_gemm_gated_ws(bb, D, L->wg, L->wu, F, gate, up, act, B * Tp, D, gs, gs_bytes, s);
    if (rc) return rc;
    if (ln_next && a_next)
        return launch_gemm_norm_ws(act, F, L->wd, L->y, D, h1, D, B * Tp, D, F, ln_next, L->eps, a_next, D, gs,
                                   gs_bytes, s);
    return launch_gemm_ws(act, F, L->wd, L->y, D, h1, D, B * Tp, D, F, nullptr, gs, gs_bytes, s);
}

int vitcop_decoder_layer_prefill(const vitcop_decoder_layer_t* L, void* ws, size_t ws_bytes, void* stream) {
    return decoder_layer_run(L, nullptr, nullptr, nullptr, ws, ws_bytes, stream);
}

static vitcop_decoder_layer_t first_decoder_layer(const vitcop_decoder_schedule_t* S) {
    vitcop_decoder_layer_t L{};
    L.B = S->B; L.T = S->T; L.D = S->D; L.Hq = S->Hq; L.Hkv = S->Hkv; L.d = S->d; L.F = S->F;
    L.vis_start = S->vis_start; L.n_vis = S->n_vis; L.keep = S->n_vis; L.eps = S->eps; L.theta = S->theta;
    return L;
}

static int check_decoder_schedule(const vitcop_decoder_schedule_t* S) {
    REQUIRE(S, VITCOP_EINVAL, "decoder_schedule: descriptor is null");
    REQUIRE(S->n_layers >= 1 && S->n_stages >= 0, VITCOP_EINVAL, "decoder_schedule: n_layers=%d n_stages=%d",
            S->n_layers, S->n_stages);
    REQUIRE(S->n_stages == 0 || (S->prune_layer && S->prune_keep), VITCOP_EINVAL,
            "decoder_schedule: null stage arrays");
    int prev_layer = -1, prev_keep = S->n_vis;
    for (int i = 0; i < S->n_stages; ++i) {
        REQUIRE(S->prune_layer[i] > prev_layer && S->prune_layer[i] < S->n_layers, VITCOP_EINVAL,
                "decoder_schedule: stage %d at layer %d (must ascend within [0,%d))", i, S->prune_layer[i],
                S->n_layers);
        REQUIRE(S->prune_keep[i] >= 0 && S->prune_keep[i] <= prev_keep, VITCOP_EINVAL,
                "decoder_schedule: stage %d keeps %d of %d", i, S->prune_keep[i], prev_keep);
        prev_layer = S->prune_layer[i];
        prev_keep = S->prune_keep[i];
    }
    const vitcop_decoder_layer_t L = first_decoder_layer(S);
    return check_decoder_layer(&L);
}

size_t vitcop_decoder_schedule_workspace_bytes(const vitcop_decoder_schedule_t* S) {
    if (check_decoder_schedule(S) != VITCOP_OK) return 0;
    vitcop_decoder_layer_t L = first_decoder_layer(S);
    size_t layer_max = 0;         // the largest layer workspace along the schedule
    int stage = 0;
    for (int l = 0; l < S->n_layers; ++l) {
        L.keep = L.n_vis;
        const bool prune_here = stage < S->n_stages && S->prune_layer[stage] == l;
        if (prune_here) L.keep = S->prune_keep[stage++];
        layer_max = std::max(layer_max, vitcop_decoder_layer_workspace_bytes(&L));
        L.T = L.T - L.n_vis + L.keep;
        L.n_vis = L.keep;
    }
    const size_t B = S->B, T = S->T, D = S->D;
    return layer_max + 4 * up256(B * T * D * 2) + 2 * up256(B * T * 4);      // hidden and normalised, ping-pong
}

// State carried from layer to layer of a whole-model run, and the ping-pong buffers it lives in.
struct DecoderRun {
    const uint16_t* h;            // hidden state entering the next layer
    const uint16_t* a_pre;        // its RMSNorm with that layer's ln1, if the layer before left it
    const int32_t* pos;
    int cur_T, cur_vis, stage, pp;
    uint16_t* hbuf[2];
    uint16_t* abuf[2];
    int32_t* pbuf[2];
    void* lws;
    size_t lws_bytes;
    // a right-padded batch (after Stage II): the samples' visual counts on the device while they differ,
    // their host mirror, two buffers for the counts after a pruning layer, and the real cache lengths
    const int32_t* nv_dev = nullptr;
    int* nv_host = nullptr;
    int32_t* nvbuf[2] = {nullptr, nullptr};
    int nvpp = 0;
    int* cache_len = nullptr;     // host, [n_layers * B], may be null
};

// Layers [l_begin, l_end) of S; a Stage III budget above the visual tokens still present keeps them all.
static int run_decoder_layers(const vitcop_decoder_schedule_t* S, int l_begin, int l_end, DecoderRun& r,
                              void* stream) {
    for (int l = l_begin; l < l_end; ++l) {
        vitcop_decoder_layer_t L = first_decoder_layer(S);
        L.T = r.cur_T; L.n_vis = r.cur_vis; L.keep = r.cur_vis;
        L.h = r.h; L.positions = r.pos;
        L.ln1 = S->ln1[l]; L.ln2 = S->ln2[l]; L.wq = S->wq[l]; L.wk = S->wk[l]; L.wv = S->wv[l]; L.wo = S->wo[l];
        L.wg = S->wg[l]; L.wu = S->wu[l]; L.wd = S->wd[l];
        const bool last = l + 1 == S->n_layers;
        const bool prune_here = r.stage < S->n_stages && S->prune_layer[r.stage] == l;
        if (prune_here) {
            if (S->stage_norms) L.norms = S->stage_norms[r.stage];
            if (S->stage_keep_idx) L.keep_idx = S->stage_keep_idx[r.stage];
            L.keep = std::min(S->prune_keep[r.stage++], r.cur_vis);
            L.positions_out = r.pbuf[r.pp];
            if (r.nv_dev) {
                L.n_vis_samples = r.nv_dev;
                L.n_vis_samples_out = r.nvbuf[r.nvpp];
            }
        }
        L.y = last ? S->y_out : r.hbuf[l & 1];
        if (S->k_cache && S->v_cache) {
            L.k_cache = S->k_cache[l];
            L.v_cache = S->v_cache[l];
            L.cache_capacity = S->cache_capacity;
        }
        const uint16_t* ln_next = last ? nullptr : static_cast<const uint16_t*>(S->ln1[l + 1]);
        int rc = decoder_layer_run(&L, r.a_pre, ln_next, r.abuf[l & 1], r.lws, r.lws_bytes, stream);
        if (rc) return rc;
        r.a_pre = ln_next ? r.abuf[l & 1] : nullptr;
        if (prune_here) {
            r.pos = r.pbuf[r.pp];
            r.pp ^= 1;
            if (r.nv_dev && L.keep < r.cur_vis) {      // the selection ran and wrote the new counts
                bool differ = false;
                for (int b = 0; b < S->B; ++b) {
                    r.nv_host[b] = std::min(r.nv_host[b], L.keep);
                    differ |= r.nv_host[b] != L.keep;
                }
                r.nv_dev = differ ? r.nvbuf[r.nvpp] : nullptr;
                r.nvpp ^= 1;
            }
            r.cur_T = r.cur_T - r.cur_vis + L.keep;
            r.cur_vis = L.keep;
        }
        if (r.cache_len)
            for (int b = 0; b < S->B; ++b)
                r.cache_len[(size_t)l * S->B + b] = r.cur_T - (r.nv_dev ? r.cur_vis - r.nv_host[b] : 0);
        r.h = L.y;
    }
    return VITCOP_OK;
}

int vitcop_decoder_schedule_prefill(const vitcop_decoder_schedule_t* S, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_decoder_schedule(S);
    if (rc) return rc;
    REQUIRE(S->h && S->positions && S->y_out && S->ln1 && S->ln2 && S->wq && S->wk && S->wv && S->wo && S->wg &&
                S->wu && S->wd,
            VITCOP_EINVAL, "decoder_schedule: null pointer");
    const size_t need = vitcop_decoder_schedule_workspace_bytes(S);
    REQUIRE(ws && ws_bytes >= need, VITCOP_EWORKSPACE, "decoder_schedule: workspace needs %zu bytes", need);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t B = S->B, T = S->T, D = S->D;
    Carver c(ws);
    DecoderRun r{S->h, nullptr, S->positions, S->T, S->n_vis, 0, 0, {}, {}, {}, nullptr, 0};
    for (int i = 0; i < 2; ++i) r.hbuf[i] = c.take<uint16_t>(B * T * D * 2);
    for (int i = 0; i < 2; ++i) r.abuf[i] = c.take<uint16_t>(B * T * D * 2);
    for (int i = 0; i < 2; ++i) r.pbuf[i] = c.take<int32_t>(B * T * 4);
    r.lws = c.base + c.used;
    r.lws_bytes = ws_bytes - c.used;
    rc = run_decoder_layers(S, 0, S->n_layers, r, stream);
    if (rc) return rc;
    if (S->positions_out) {
        rc = hip_status(hipMemcpyAsync(S->positions_out, r.pos, (size_t)B * r.cur_T * 4, hipMemcpyDeviceToDevice, s),
                        "copy positions");
    }
    return rc;
}

/* ------------------------------------------- whole procedure with Stage II */

// The sequences after Stage II, right-padded to T_new rows: text before the visual block unchanged, row j of
// the new visual block = row j of Stage II's output with the position of its representative token, the text
// after it, then zero rows (position 0) up to the longest sample.  One workgroup per output row.
__global__ __launch_bounds__(256) void stage2_splice_kernel(
    const uint16_t* __restrict__ h, const uint16_t* __restrict__ out_feats, const int32_t* __restrict__ pos,
    const int32_t* __restrict__ out_index, const int32_t* __restrict__ n_out, int T, int D, int vis_start,
    int n_vis, int T_new, uint16_t* __restrict__ h_new, int32_t* __restrict__ pos_new) {
    const int j = blockIdx.x, b = blockIdx.y;
    const int no = n_vis > 0 ? n_out[b] : 0;
    const uint16_t* src = nullptr;
    int pos_src = -1;
    if (j < vis_start) {
        src = h + ((int64_t)b * T + j) * D;
        pos_src = j;
    } else if (j < vis_start + no) {
        src = out_feats + ((int64_t)b * n_vis + (j - vis_start)) * D;
        pos_src = vis_start + out_index[(int64_t)b * n_vis + (j - vis_start)];
    } else if (j < T - n_vis + no) {
        pos_src = j - no + n_vis;
        src = h + ((int64_t)b * T + pos_src) * D;
    }
    uint4* dst = reinterpret_cast<uint4*>(h_new + ((int64_t)b * T_new + j) * D);
    const uint4* s4 = reinterpret_cast<const uint4*>(src);
    for (int c = threadIdx.x; c < D / 8; c += blockDim.x) dst[c] = src ? s4[c] : make_uint4(0, 0, 0, 0);
    if (threadIdx.x == 0) pos_new[(int64_t)b * T_new + j] = pos_src >= 0 ? pos[(int64_t)b * T + pos_src] : 0;
}

static int check_full_schedule(const vitcop_full_schedule_t* F) {
    REQUIRE(F, VITCOP_EINVAL, "full_schedule: descriptor is null");
    const vitcop_decoder_schedule_t* S = &F->S;
    int rc = check_decoder_schedule(S);
    if (rc) return rc;
    REQUIRE(F->stage2_layer >= 0 && F->stage2_layer < S->n_layers, VITCOP_EINVAL, "full_schedule: stage2_layer=%d",
            F->stage2_layer);
    REQUIRE(S->n_stages == 0 || S->prune_layer[0] > F->stage2_layer, VITCOP_EINVAL,
            "full_schedule: Stage III layers must come after layer %d", F->stage2_layer);
    REQUIRE(F->stage2_budget >= 0 && F->stage2_budget <= S->n_vis, VITCOP_EINVAL, "full_schedule: stage2_budget=%d",
            F->stage2_budget);
    return check_vic(S->B, S->n_vis, S->D, F->d_c, F->tau, F->n_centers);
}

// Stage II scratch: the spliced hidden states, the normalised input, K of all tokens, norm partials, the
// identity keep list the norm pass writes, norms, labels, cluster counts, the new visual blocks, their
// representatives, their sizes (twice more for the counts after later stages); then the two stages' own.
static size_t full_schedule_stage2_bytes(const vitcop_full_schedule_t* F) {
    const vitcop_decoder_schedule_t* S = &F->S;
    const size_t B = S->B, T = S->T, D = S->D, n = S->n_vis, kd = (size_t)S->Hkv * S->d;
    size_t b = up256(B * T * D * 2) + up256(B * T * D * 2) + up256(B * T * kd * 2) +
               up256((size_t)gemm_sumsq_parts((int)kd) * B * T * 4) + up256(B * T * 4);
    b += 2 * up256(B * n * 4) + 4 * up256(B * 4) + up256(B * n * D * 2) + up256(B * n * 4);
    b += up256(vic_workspace_bytes((int)B, (int)n)) + up256(collab_workspace_bytes((int)B, (int)n));
    b += up256(gemm_workspace_bytes((int)(B * T), (int)kd, (int)D));
    return b;
}

size_t vitcop_full_schedule_workspace_bytes(const vitcop_full_schedule_t* F) {
    if (check_full_schedule(F) != VITCOP_OK) return 0;
    return vitcop_decoder_schedule_workspace_bytes(&F->S) + full_schedule_stage2_bytes(F);
}

int vitcop_full_schedule_prefill(const vitcop_full_schedule_t* F, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_full_schedule(F);
    if (rc) return rc;
    const vitcop_decoder_schedule_t* S = &F->S;
    REQUIRE(S->h && S->positions && S->y_out && S->ln1 && S->ln2 && S->wq && S->wk && S->wv && S->wo && S->wg &&
                S->wu && S->wd && F->vis_xy && F->T_final,
            VITCOP_EINVAL, "full_schedule: null pointer");
    const size_t need = vitcop_full_schedule_workspace_bytes(F);
    REQUIRE(ws && ws_bytes >= need, VITCOP_EWORKSPACE, "full_schedule: workspace needs %zu bytes", need);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t B = S->B, T = S->T, D = S->D, n = S->n_vis, kd = (size_t)S->Hkv * S->d;
    const int vs = S->vis_start, P = gemm_sumsq_parts((int)kd), ls = F->stage2_layer;
    Carver c(ws);
    DecoderRun r{S->h, nullptr, S->positions, S->T, S->n_vis, 0, 0, {}, {}, {}, nullptr, 0};
    for (int i = 0; i < 2; ++i) r.hbuf[i] = c.take<uint16_t>(B * T * D * 2);
    for (int i = 0; i < 2; ++i) r.abuf[i] = c.take<uint16_t>(B * T * D * 2);
    for (int i = 0; i < 2; ++i) r.pbuf[i] = c.take<int32_t>(B * T * 4);
    uint16_t* h_new = c.take<uint16_t>(B * T * D * 2);
    uint16_t* a_all = c.take<uint16_t>(B * T * D * 2);
    uint16_t* k_all = c.take<uint16_t>(B * T * kd * 2);
    float* parts = c.take<float>((size_t)P * B * T * 4);
    int32_t* idx_all = c.take<int32_t>(B * T * 4);
    float* norms = c.take<float>(B * n * 4);
    int32_t* labels = c.take<int32_t>(B * n * 4);
    int32_t* n_clusters = c.take<int32_t>(B * 4);
    int32_t* n_out_dev = c.take<int32_t>(B * 4);
    for (int i = 0; i < 2; ++i) r.nvbuf[i] = c.take<int32_t>(B * 4);
    uint16_t* out_feats = c.take<uint16_t>(B * n * D * 2);
    int32_t* out_index = c.take<int32_t>(B * n * 4);
    void* vic_ws = c.take<char>(vic_workspace_bytes((int)B, (int)n));
    void* collab_ws = c.take<char>(collab_workspace_bytes((int)B, (int)n));
    const size_t gs_bytes = gemm_workspace_bytes((int)(B * T), (int)kd, (int)D);
    void* gs = c.take<char>(gs_bytes);
    r.lws = c.base + c.used;
    r.lws_bytes = ws_bytes - c.used;
    r.cache_len = F->cache_len_samples;

    rc = run_decoder_layers(S, 0, ls, r, stream);
    if (rc) return rc;

    // Stage II on entry to layer ls.  K-norms of that layer (Eq. 4): K of the normalised input with the
    // squared norms as a side output; keeping all n_vis tokens makes the selection pass write the norms.
    const uint16_t* a = r.a_pre;
    if (!a) {
        rc = launch_rmsnorm(r.h, D, S->ln1[ls], S->eps, a_all, D, (int)(B * T), (int)D, s);
        if (rc) return rc;
        a = a_all;
    }
    rc = launch_gemm_ws(a, D, S->wk[ls], k_all, kd, nullptr, 0, (int)(B * T), (int)kd, (int)D, parts, gs, gs_bytes, s);
    if (rc) return rc;
    rc = launch_select_smallest(parts, P, (int64_t)(B * T), T, vs, 1, norms, (int)B, (int)T, vs, (int)n, (int)n,
                                idx_all, s);
    if (rc) return rc;
    const uint16_t* feats = r.h + (size_t)vs * D;
    std::vector<int> n_out(B, 0);
    if (n > 0) {
        rc = launch_vic(feats, D, (int64_t)T * D, F->vis_xy, (int)B, (int)n, (int)D, F->d_c, F->tau, F->n_centers,
                        labels, n_clusters, nullptr, nullptr, nullptr, nullptr, vic_ws, s);
        if (rc) return rc;
        rc = launch_collab(feats, D, (int64_t)T * D, labels, n_clusters, norms, (int)B, (int)n, (int)D,
                           F->stage2_budget, out_feats, out_index, n_out_dev, nullptr, collab_ws, s);
        if (rc) return rc;
        rc = hip_status(hipMemcpyAsync(n_out.data(), n_out_dev, B * 4, hipMemcpyDeviceToHost, s),
                        "read Stage II counts");
        if (rc) return rc;
    }
    rc = hip_status(hipStreamSynchronize(s), "hipStreamSynchronize");
    if (rc) return rc;
    int n_max = 0;
    bool differ = false;
    for (size_t b = 0; b < B; ++b) {
        REQUIRE(n_out[b] >= 0 && (size_t)n_out[b] <= n, VITCOP_EHIP, "full_schedule: Stage II returned %d tokens",
                n_out[b]);
        n_max = std::max(n_max, n_out[b]);
        differ |= n_out[b] != n_out[0];
        if (F->n_stage2) F->n_stage2[b] = n_out[b];
    }
    auto copy = [&](void* dst, const void* src, size_t bytes) {
        if (rc == VITCOP_OK && dst && bytes)
            rc = hip_status(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, s), "copy after Stage II");
    };
    copy(F->labels, labels, B * n * 4);
    copy(F->norms, norms, B * n * 4);
    copy(F->out_index, out_index, B * n * 4);
    if (rc) return rc;
    // the new sequences: text, new visual block, text, padding up to the longest sample
    const size_t T_new = T - n + (size_t)n_max;
    int32_t* pos_new = r.pbuf[r.pp];
    hipLaunchKernelGGL(stage2_splice_kernel, dim3((unsigned)T_new, (unsigned)B), dim3(256), 0, s, r.h, out_feats,
                       r.pos, out_index, n_out_dev, (int)T, (int)D, vs, (int)n, (int)T_new, h_new, pos_new);
    rc = launch_status("stage2_splice");
    if (rc) return rc;
    r.h = h_new;
    r.a_pre = nullptr;
    r.pos = pos_new;
    r.pp ^= 1;
    r.cur_T = (int)T_new;
    r.cur_vis = n_max;
    r.nv_host = n_out.data();
    r.nv_dev = differ ? n_out_dev : nullptr;

    rc = run_decoder_layers(S, ls, S->n_layers, r, stream);
    if (rc) return rc;
    *F->T_final = r.cur_T;
    if (F->T_final_samples)
        for (size_t b = 0; b < B; ++b) F->T_final_samples[b] = r.cur_T - (r.nv_dev ? r.cur_vis - n_out[b] : 0);
    if (S->positions_out) {
        rc = hip_status(hipMemcpyAsync(S->positions_out, r.pos, B * (size_t)r.cur_T * 4, hipMemcpyDeviceToDevice, s),
                        "copy positions");
    }
    return rc;
}

/* ------------------------------------------------------------- decode step */

static int check_decode(int B, int N, int Hq, int Hkv, int d) {
    REQUIRE(B >= 0 && N >= 1 && Hq >= 1 && Hkv >= 1, VITCOP_EINVAL, "decode_attn: B=%d N=%d Hq=%d Hkv=%d", B, N, Hq, Hkv);
    REQUIRE(Hq % Hkv == 0, VITCOP_EINVAL, "decode_attn: Hq=%d not a multiple of Hkv=%d", Hq, Hkv);
    REQUIRE(d == 64 || d == 128, VITCOP_EUNSUPPORTED, "decode_attn: d=%d (64 or 128)", d);
    REQUIRE(Hkv <= 65535 && B <= 65535, VITCOP_EUNSUPPORTED, "decode_attn: Hkv or B above 65535");
    REQUIRE((long)N * Hkv * d < (1L << 31), VITCOP_EUNSUPPORTED, "decode_attn: one sample's cache must stay below 2^31 elements");
    return VITCOP_OK;
}

size_t vitcop_decode_attn_workspace_bytes(int B, int N, int Hq, int Hkv, int d) {
    if (check_decode(B, N, Hq, Hkv, d) != VITCOP_OK) return 0;
    return decode_workspace_bytes(B, N, Hq, Hkv, d);
}

int vitcop_decode_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out, float* lse_out,
                       int B, int N, int Hq, int Hkv, int d, float scale, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_decode(B, N, Hq, Hkv, d);
    if (rc) return rc;
    REQUIRE(std::isfinite(scale) && scale >= 0.f, VITCOP_EINVAL, "decode_attn: scale");
    if (B == 0) return VITCOP_OK;
    REQUIRE(q && k && v && out, VITCOP_EINVAL, "decode_attn: null pointer");
    REQUIRE(aligned16(q) && aligned16(k) && aligned16(v) && aligned16(out), VITCOP_EINVAL,
            "decode_attn: pointers must be 16-byte aligned");
    const size_t need = decode_workspace_bytes(B, N, Hq, Hkv, d);
    REQUIRE(ws && ws_bytes >= need, VITCOP_EWORKSPACE, "decode_attn: workspace %zu < %zu", ws_bytes, need);
    if (scale == 0.f) scale = 1.0f / std::sqrt((float)d);
    return launch_decode_attn(q, k, v, out, lse_out, B, N, Hq, Hkv, d, scale, ws, static_cast<hipStream_t>(stream));
}

/* ------------------------------------------------ whole-model decoding step */

static int check_decoder_decode(const vitcop_decoder_decode_t* S) {
    REQUIRE(S, VITCOP_EINVAL, "decoder_decode: descriptor is null");
    REQUIRE(S->B >= 1 && S->D >= 32 && S->Hq >= 1 && S->Hkv >= 1 && S->F >= 32 && S->n_layers >= 1, VITCOP_EINVAL,
            "decoder_decode: B=%d D=%d Hq=%d Hkv=%d F=%d n_layers=%d", S->B, S->D, S->Hq, S->Hkv, S->F, S->n_layers);
    REQUIRE(S->B <= 256, VITCOP_EUNSUPPORTED, "decoder_decode: B=%d above 256", S->B);
    REQUIRE(S->Hq % S->Hkv == 0, VITCOP_EINVAL, "decoder_decode: Hq=%d not a multiple of Hkv=%d", S->Hq, S->Hkv);
    REQUIRE(S->d == 64 || S->d == 128, VITCOP_EUNSUPPORTED, "decoder_decode: d=%d (64 or 128)", S->d);
    REQUIRE(S->D % 64 == 0 && S->F % 128 == 0 && (S->Hq * S->d) % 64 == 0, VITCOP_EUNSUPPORTED,
            "decoder_decode: D=%d must be a multiple of 64, F=%d of 128", S->D, S->F);
    REQUIRE(std::isfinite(S->eps) && S->eps >= 0.f && std::isfinite(S->theta) && S->theta > 1.f, VITCOP_EINVAL,
            "decoder_decode: eps or theta");
    REQUIRE(S->n_cached, VITCOP_EINVAL, "decoder_decode: n_cached is null");
    for (int l = 0; l < S->n_layers; ++l) {
        REQUIRE(S->n_cached[l] >= 0 && S->n_cached[l] < S->cache_capacity, VITCOP_EINVAL,
                "decoder_decode: layer %d holds %d tokens, capacity %d", l, S->n_cached[l], S->cache_capacity);
        const int rc = check_decode(S->B, S->n_cached[l] + 1, S->Hq, S->Hkv, S->d);
        if (rc) return rc;
    }
    REQUIRE((long)S->cache_capacity * S->Hkv * S->d < (1L << 31), VITCOP_EUNSUPPORTED,
            "decoder_decode: one sample's cache must stay below 2^31 elements");
    return VITCOP_OK;
}

static size_t decoder_decode_gemm_scratch(const vitcop_decoder_decode_t* S) {
    const int B = S->B, D = S->D, qd = S->Hq * S->d, kd = S->Hkv * S->d, F = S->F;
    size_t n = gemm_workspace_bytes(B, qd + 2 * kd, D);
    n = std::max(n, gemm_workspace_bytes(B, D, qd));
    n = std::max(n, gemm_workspace_bytes(B, 2 * F, D));
    return std::max(n, gemm_workspace_bytes(B, D, F));
}

size_t vitcop_decoder_decode_workspace_bytes(const vitcop_decoder_decode_t* S) {
    if (check_decoder_decode(S) != VITCOP_OK) return 0;
    const size_t B = S->B, D = S->D, qd = (size_t)S->Hq * S->d, kd = (size_t)S->Hkv * S->d, F = S->F;
    int n_max = 0;
    for (int l = 0; l < S->n_layers; ++l) n_max = std::max(n_max, S->n_cached[l] + 1);
    size_t n = 6 * up256(B * D * 2);                                     // a (two), hidden (two), h1, b
    n += 2 * up256(B * qd * 2) + 2 * up256(B * kd * 2);                  // q, attention output, new K and V
    n += 3 * up256(B * F * 2);                                           // gate, up, activation
    n += up256(decode_workspace_bytes((int)B, n_max, S->Hq, S->Hkv, S->d));
    return n + up256(decoder_decode_gemm_scratch(S));
}

int vitcop_decoder_decode_step(const vitcop_decoder_decode_t* S, void* ws, size_t ws_bytes, void* stream) {
    int rc = check_decoder_decode(S);
    if (rc) return rc;
    REQUIRE(S->h && S->positions && S->y_out && S->ln1 && S->ln2 && S->wq && S->wk && S->wv && S->wo && S->wg &&
                S->wu && S->wd && S->k_cache && S->v_cache,
            VITCOP_EINVAL, "decoder_decode: null pointer");
    const size_t need = vitcop_decoder_decode_workspace_bytes(S);
    REQUIRE(ws && ws_bytes >= need, VITCOP_EWORKSPACE, "decoder_decode: workspace needs %zu bytes", need);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int B = S->B, D = S->D, qd = S->Hq * S->d, kd = S->Hkv * S->d, F = S->F;
    int n_max = 0;
    for (int l = 0; l < S->n_layers; ++l) n_max = std::max(n_max, S->n_cached[l] + 1);
    Carver c(ws);
    uint16_t* abuf[2] = {c.take<uint16_t>((size_t)B * D * 2), c.take<uint16_t>((size_t)B * D * 2)};
    uint16_t* hbuf[2] = {c.take<uint16_t>((size_t)B * D * 2), c.take<uint16_t>((size_t)B * D * 2)};
    uint16_t* h1 = c.take<uint16_t>((size_t)B * D * 2);
    uint16_t* bb = c.take<uint16_t>((size_t)B * D * 2);
    uint16_t* qb = c.take<uint16_t>((size_t)B * qd * 2);
    uint16_t* ob = c.take<uint16_t>((size_t)B * qd * 2);
    uint16_t* k_new = c.take<uint16_t>((size_t)B * kd * 2);
    uint16_t* v_new = c.take<uint16_t>((size_t)B * kd * 2);
    uint16_t* gate = c.take<uint16_t>((size_t)B * F * 2);
    uint16_t* up = c.take<uint16_t>((size_t)B * F * 2);
    uint16_t* act = c.take<uint16_t>((size_t)B * F * 2);
    void* dws = c.take<char>(decode_workspace_bytes(B, n_max, S->Hq, S->Hkv, S->d));
    const size_t gs_bytes = decoder_decode_gemm_scratch(S);
    void* gs = c.take<char>(gs_bytes);

    const uint16_t* h = S->h;
    if (gemv_applies(B, D) && gemv_applies(B, qd) && gemv_applies(B, F) && S->d % 2 == 0) {
        // a handful of rows: every product is a stream over its weights, with the norms, the rotary embedding,
        // the cache append, the activation and the residual adds inside the streaming kernels
        const int64_t kv_batch = (int64_t)S->cache_capacity * kd;
        for (int l = 0; l < S->n_layers; ++l) {
            REQUIRE(S->ln1[l] && S->ln2[l] && S->wq[l] && S->wk[l] && S->wv[l] && S->wo[l] && S->wg[l] && S->wu[l] &&
                        S->wd[l] && S->k_cache[l] && S->v_cache[l],
                    VITCOP_EINVAL, "decoder_decode: layer %d has a null pointer", l);
            const int N = S->n_cached[l];
            // per-sample cache lengths: the append row and the keys attended over come from the device array
            const int32_t* ncs = S->n_cached_samples ? S->n_cached_samples + (size_t)l * B : nullptr;
            const size_t row0 = ncs ? 0 : (size_t)N * kd;
            rc = launch_gemv_qkv_rope(h, D, S->ln1[l], S->eps, S->wq[l], S->wk[l], S->wv[l], qb,
                                      S->k_cache[l] + row0, S->v_cache[l] + row0, kv_batch,
                                      S->positions, B, S->Hq, S->Hkv, S->d, D, S->theta, s, ncs);
            if (rc) return rc;
            // (one sample and few slices: the output projection combines them itself, no merge launch; with more
            // samples every workgroup would repeat the combination for each of them and the launch is cheaper)
            DecodeParts slices{nullptr, nullptr, 0};
            rc = launch_decode_attn(qb, S->k_cache[l], S->v_cache[l], ob, nullptr, B, N + 1, S->Hq, S->Hkv, S->d,
                                    1.0f / std::sqrt((float)S->d), dws, s, kv_batch, B == 1 ? &slices : nullptr, ncs);
            if (rc) return rc;
            rc = launch_gemv(ob, qd, nullptr, 0.f, S->wo[l], h1, D, h, D, B, D, qd, s, &slices, S->d);
            if (rc) return rc;
            rc = launch_gemv_gated(h1, D, S->ln2[l], S->eps, S->wg[l], S->wu[l], act, F, B, F, D, s);
            if (rc) return rc;
            uint16_t* y = l + 1 == S->n_layers ? S->y_out : hbuf[l & 1];
            rc = launch_gemv(act, F, nullptr, 0.f, S->wd[l], y, D, h1, D, B, D, F, s);
            if (rc) return rc;
            h = y;
        }
        return VITCOP_OK;
    }
    const uint16_t* a = nullptr;            // RMSNorm of h with this layer's ln1, left by the layer before
    for (int l = 0; l < S->n_layers; ++l) {
        REQUIRE(S->ln1[l] && S->ln2[l] && S->wq[l] && S->wk[l] && S->wv[l] && S->wo[l] && S->wg[l] && S->wu[l] &&
                    S->wd[l] && S->k_cache[l] && S->v_cache[l],
                VITCOP_EINVAL, "decoder_decode: layer %d has a null pointer", l);
        const int N = S->n_cached[l];
        const bool last = l + 1 == S->n_layers;
        if (!a) {
            rc = launch_rmsnorm(h, D, S->ln1[l], S->eps, abuf[0], D, B, D, s);
            if (rc) return rc;
            a = abuf[0];
        }
        const uint16_t* const w3[3] = {S->wk[l], S->wq[l], S->wv[l]};
        uint16_t* const y3[3] = {k_new, qb, v_new};
        const int n3[3] = {kd, qd, kd};
        rc = launch_gemm_triple_ws(a, D, w3, y3, n3, B, D, gs, gs_bytes, s);
        if (rc) return rc;
        // the rotary embedding; the new token's K and V become row N of every sample's cache
        const int32_t* ncs = S->n_cached_samples ? S->n_cached_samples + (size_t)l * B : nullptr;
        const size_t row0 = ncs ? 0 : (size_t)N * kd;
        rc = launch_rope_append(qb, k_new, v_new, S->positions, B, S->Hq, S->Hkv, S->d, S->theta,
                                S->k_cache[l] + row0, S->v_cache[l] + row0, (int64_t)S->cache_capacity * kd, s, ncs);
        if (rc) return rc;
        rc = launch_decode_attn(qb, S->k_cache[l], S->v_cache[l], ob, nullptr, B, N + 1, S->Hq, S->Hkv, S->d,
                                1.0f / std::sqrt((float)S->d), dws, s, (int64_t)S->cache_capacity * kd, nullptr, ncs);
        if (rc) return rc;
        rc = launch_gemm_norm_ws(ob, qd, S->wo[l], h1, D, h, D, B, D, qd, S->ln2[l], S->eps, bb, D, gs, gs_bytes, s);
        if (rc) return rc;
        rc = launch_gemm_gated_ws(bb, D, S->wg[l], S->wu[l], F, gate, up, act, B, D, gs, gs_bytes, s);
        if (rc) return rc;
        uint16_t* y = last ? S->y_out : hbuf[l & 1];
        if (!last && S->ln1[l + 1]) {
            uint16_t* a_next = abuf[(l + 1) & 1];
            rc = launch_gemm_norm_ws(act, F, S->wd[l], y, D, h1, D, B, D, F, S->ln1[l + 1], S->eps, a_next, D, gs,
                                     gs_bytes, s);
            a = a_next;
        } else {
            rc = launch_gemm_ws(act, F, S->wd[l], y, D, h1, D, B, D, F, nullptr, gs, gs_bytes, s);
            a = nullptr;
        }
        if (rc) return rc;
        h = y;
    }
    return VITCOP_OK;
}

#pragma GCC visibility pop
}  // extern "C"
