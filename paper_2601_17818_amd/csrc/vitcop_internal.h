// Internal declarations shared by the translation units of libvitcop.
// Host-side argument checking lives in api.cpp; each *.hip file owns its
// kernels and exposes one or two launch functions declared here.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "vitcop.h"

namespace vitcop {

static inline size_t up256(size_t n) { return (n + 255) & ~(size_t)255; }

// Records a thread-local message and returns `code` (a VITCOP_E* value).
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
// VITCOP_OK, or records the HIP error text and returns VITCOP_EHIP.
int hip_status(hipError_t e, const char* what);
int launch_status(const char* kernel_name);

// ---- K-norm + selection (knorm_select.hip) -------------------------------
int launch_knorm(const uint16_t* k, int64_t row_stride, int64_t batch_stride, int B,
                 int row_elems, int vis_start, int n_vis, float* norms, hipStream_t s);
// Ranks the n_vis candidates of each sample and writes the keep list.
// value(b,i) = sum_{p<n_parts} parts[p*part_stride + b*sample_stride + offset + i];
// do_sqrt: rank sqrt(value); norms_out (nullable) receives the ranked values.
int launch_select_smallest(const float* parts, int n_parts, int64_t part_stride,
                           int64_t sample_stride, int64_t offset, int do_sqrt,
                           float* norms_out, int B, int T, int vis_start, int n_vis,
                           int keep, int32_t* keep_idx, hipStream_t s,
                           const int32_t* n_vis_samples = nullptr, int32_t* n_vis_samples_out = nullptr);

// ---- compaction (compact.hip) --------------------------------------------
int launch_compact(const vitcop_gather_t* t, int n, const int32_t* idx, int B, int T_out,
                   hipStream_t s);

// ---- Stage I filter (filter.hip) -----------------------------------------
int launch_filter(const uint16_t* q_cls, const uint16_t* k, int B, int N, int H, int d,
                  int keep, float scale, float* scores_out, int32_t* idx_out,
                  float* logits_ws, hipStream_t s);
// Device address of the library-owned scratch array of FILTER_STATIC_SCRATCH_BYTES on the current device.
constexpr size_t FILTER_STATIC_SCRATCH_BYTES = VITCOP_FILTER_STATIC_MAX_BYTES;
int filter_static_scratch(float** out);

// ---- attention (attn.hip) -------------------------------------------------
int launch_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                float* lse, int B, int N, int Hq, int Hkv, int d, float scale, int causal,
                hipStream_t s);

// ---- projection GEMM (gemm.hip) -------------------------------------------
int gemm_sumsq_parts(int N);
int launch_gemm(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y,
                int64_t y_stride, const uint16_t* res, int64_t res_stride, int M, int N,
                int K, float* sumsq_parts, hipStream_t s);
// y1 = x W1^T [M,N1] and y2 = x W2^T [M,N2] (dense outputs), one launch when the shapes allow
int launch_gemm_pair(const uint16_t* x, int64_t x_stride, const uint16_t* w1, uint16_t* y1, int N1,
                     const uint16_t* w2, uint16_t* y2, int N2, int M, int K, hipStream_t s);

// The same two calls with a scratch buffer: launches with few rows (M <= 256) then stream the weights
// through a split-K kernel (gemm_skinny.hip) whose fp32 partials live in `ws`; with ws == nullptr, too
// small a buffer or any other shape they are the calls above.  gemm_workspace_bytes is what the
// split-K path of one launch (N = N1 + N2 for a pair) needs, 0 if it does not apply.
size_t gemm_workspace_bytes(int M, int N, int K);
int launch_gemm_ws(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y, int64_t y_stride,
                   const uint16_t* res, int64_t res_stride, int M, int N, int K, float* sumsq_parts, void* ws,
                   size_t ws_bytes, hipStream_t s);
// y = x W^T + res as launch_gemm_ws, and norm_out = RMSNorm(y) * ln_w (rows norm_stride apart): fused
// into the few-row path's reduction where that applies, otherwise the projection and launch_rmsnorm.
int launch_gemm_norm_ws(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y, int64_t y_stride,
                        const uint16_t* res, int64_t res_stride, int M, int N, int K, const uint16_t* ln_w,
                        float eps, uint16_t* norm_out, int64_t norm_stride, void* ws, size_t ws_bytes,
                        hipStream_t s);
// Three projections of the same input (dense outputs [M, n[i]]): one launch on the few-row path when
// it applies and n[0], n[1] are multiples of 128; otherwise the first alone and the other two as a pair.
int launch_gemm_triple_ws(const uint16_t* x, int64_t x_stride, const uint16_t* const w[3], uint16_t* const y[3],
                          const int n[3], int M, int K, void* ws, size_t ws_bytes, hipStream_t s);
// out = silu(x wg^T) * (x wu^T) [M, F]: on the few-row path one launch with the activation in its
// reduction; otherwise the pair of projections into gate and up [M, F] and launch_silu_mul.
int launch_gemm_gated_ws(const uint16_t* x, int64_t x_stride, const uint16_t* wg, const uint16_t* wu, int F,
                         uint16_t* gate, uint16_t* up, uint16_t* out, int M, int K, void* ws, size_t ws_bytes,
                         hipStream_t s);
int launch_gemm_pair_ws(const uint16_t* x, int64_t x_stride, const uint16_t* w1, uint16_t* y1, int N1,
                        const uint16_t* w2, uint16_t* y2, int N2, int M, int K, void* ws, size_t ws_bytes,
                        hipStream_t s);
// k, q, v = x Wk^T, x Wq^T, x Wv^T (dense [M, Hkv d], [M, Hq d], [M, Hkv d]) with the rotary embedding of q
// and k at positions[m]: where the projections leave partial sums (few rows, or split-K of K and of the Q/V
// pair) one launch adds them up and turns q and k; otherwise launch_gemm_triple_ws and rope_kernel.
// gemm_qkv_workspace_bytes: what ws must hold for every path this may take at M rows.
size_t gemm_qkv_workspace_bytes(int M, int Hq, int Hkv, int d, int K);
int launch_gemm_qkv_rope_ws(const uint16_t* x, int64_t x_stride, const uint16_t* wk, const uint16_t* wq,
                            const uint16_t* wv, uint16_t* k, uint16_t* q, uint16_t* v, int Hq, int Hkv, int d,
                            const int32_t* positions, float theta, int M, int K, void* ws, size_t ws_bytes,
                            hipStream_t s);
// gemm_skinny.hip
// Up to three weight matrices side by side (projections of the same input in one launch): matrix i
// covers the columns [n_end[i-1], n_end[i]) of the launch (boundaries multiples of 128; unused
// entries repeat N) and writes its own output with its own row stride.
struct SkMats {
    const uint16_t* w[3];
    uint16_t* y[3];
    int64_t y_stride[3];
    int n_end[3];
};
// Where the partial sums of a launch live.  units_q > 0: the tiles of gemm_skinny_kernel
// (part[2 * workgroup + segment][m][128], workgroups by sk_first_unit over groups of upg units).
// units_q == 0: the slices of a split-K launch of the big-tile kernel, part[slice][m][n] with
// units_r slices and row stride upg.
struct SkParts {
    const float* part;
    int units_q, units_r, upg, M;
};
// k, q and v of a layer (in this order) as partial sums: for each the launch it belongs to and its first
// column there.
struct QkvParts {
    SkParts parts[3];
    int col0[3];
};
// k, q, v [M, Hkv d], [M, Hq d], [M, Hkv d] (dense) = the partial sums added in slice order and rounded to
// bf16, q and k then turned by the rotary embedding at positions[m] (rope_kernel's arithmetic).
int launch_qkv_finish(const QkvParts& P, uint16_t* k, uint16_t* q, uint16_t* v, int Hq, int Hkv, int d,
                      const int32_t* positions, float theta, hipStream_t s);

int launch_partial_reduce(const SkParts& parts, int N, const SkMats& mats, const uint16_t* res, int64_t res_stride,
                          float* sumsq_parts, const uint16_t* ln_w, float eps, uint16_t* norm_out,
                          int64_t norm_stride, uint16_t* gated_out, hipStream_t s);
bool partial_reduce_fuses_norm(int N);
// The per-slice partials of a decoding attention: part_o [B*Hq][n_splits][d] unnormalised outputs, part_ml
// [B*Hq][n_splits][2] (running maximum in log2 units, sum).  With hand_over != nullptr and at most
// DECODE_PARTS_MAX_SPLITS slices launch_decode_attn leaves the combination to the caller's next kernel
// (`out` is then not written) and describes the partials there; otherwise hand_over->part_o is null.
constexpr int DECODE_PARTS_MAX_SPLITS = 16;
struct DecodeParts {
    const float* part_o;
    const float* part_ml;
    int n_splits;
};

// gemv.hip: projections of at most GV_MAX_ROWS rows as a stream over the weights (decoding steps), with
// RMSNorm of x in the prologue (ln_w != nullptr) and the residual add, silu(gate) * up, or the rotary
// embedding with the KV-cache append in the epilogue.  N even, W dense [N][K], K within gemv_applies.
constexpr int GV_MAX_ROWS = 4;
bool gemv_applies(int B, int K);
int launch_gemv(const uint16_t* x, int64_t x_stride, const uint16_t* ln_w, float eps, const uint16_t* w, uint16_t* y,
                int64_t y_stride, const uint16_t* res, int64_t res_stride, int B, int N, int K, hipStream_t s,
                const DecodeParts* attn = nullptr, int head_dim = 0);
int launch_gemv_gated(const uint16_t* x, int64_t x_stride, const uint16_t* ln_w, float eps, const uint16_t* wg,
                      const uint16_t* wu, uint16_t* act, int64_t act_stride, int B, int F, int K, hipStream_t s);
int launch_gemv_qkv_rope(const uint16_t* x, int64_t x_stride, const uint16_t* ln_w, float eps, const uint16_t* wq,
                         const uint16_t* wk, const uint16_t* wv, uint16_t* q, uint16_t* k_dst, uint16_t* v_dst,
                         int64_t kv_batch, const int32_t* positions, int B, int Hq, int Hkv, int d, int K, float theta,
                         hipStream_t s, const int32_t* kv_rows = nullptr);

bool gemm_skinny_applies(int M, int N, int K);
size_t gemm_skinny_workspace_bytes(int M, int N, int K);
bool gemm_skinny_fuses_norm(int M, int N, int K);
int launch_gemm_skinny_gated(const uint16_t* x, int64_t x_stride, const uint16_t* wg, const uint16_t* wu, int F,
                             uint16_t* out, int M, int K, void* ws, hipStream_t s);
// (parts_out != nullptr: the rows are left as partial sums, described there, for the caller to finish;
// parts_out->part == nullptr afterwards means the launch wrote its outputs directly.)
int launch_gemm_skinny3(const uint16_t* x, int64_t x_stride, const uint16_t* const w[3], uint16_t* const y[3],
                        const int n[3], int M, int K, void* ws, hipStream_t s, SkParts* parts_out = nullptr);
int launch_gemm_skinny(const uint16_t* x, int64_t x_stride, const uint16_t* w, uint16_t* y, int64_t y_stride,
                       const uint16_t* res, int64_t res_stride, int M, int N, int K, float* sumsq_parts,
                       const uint16_t* w2, uint16_t* y2, int n_split, void* ws, hipStream_t s,
                       const uint16_t* ln_w = nullptr, float eps = 0.f, uint16_t* norm_out = nullptr,
                       int64_t norm_stride = 0);

// dist[b][i,j] = ||f_i - f_j||_2 (fp32) between the rows of each of `batch` matrices, from MFMA
// inner products and given squared row norms; sq readable and dist rows writable up to the next
// multiple of 4 entries, dist_stride % 4 == 0
int launch_pairwise_dist(const uint16_t* f, int64_t row_stride, int64_t batch_stride, const float* sq,
                         int64_t sq_batch, float* dist, int64_t dist_stride, int64_t dist_batch, int n, int K,
                         int batch, hipStream_t s);

// ---- Visual Information Clustering (vic.hip) --------------------------------
size_t vic_workspace_bytes(int B, int n);
int launch_vic(const uint16_t* feats, int64_t row_stride, int64_t batch_stride, const float* pos, int B,
               int n, int D, float d_c, float tau, int n_centers, int32_t* labels, int32_t* n_clusters,
               float* rho_out, float* delta_out, int32_t* parent_out, float* dist_out, void* ws,
               hipStream_t s);

// ---- collaborative pruning and merging (collab.hip) -------------------------
size_t collab_workspace_bytes(int B, int n);
int launch_collab(const uint16_t* feats, int64_t row_stride, int64_t batch_stride, const int32_t* labels,
                  const int32_t* n_clusters, const float* norms, int B, int n, int D, int budget,
                  uint16_t* out_feats, int32_t* out_index, int32_t* n_out, int32_t* assign, void* ws,
                  hipStream_t s);

// ---- decoder-layer pieces (decoder.hip) -------------------------------------
int launch_rmsnorm(const uint16_t* x, int64_t x_stride, const uint16_t* w, float eps, uint16_t* y,
                   int64_t y_stride, int M, int D, hipStream_t s);
// in place; q [n_tokens,Hq,d] and k [n_tokens,Hkv,d] (either may be null), positions [n_tokens]
int launch_rope(uint16_t* q, uint16_t* k, const int32_t* positions, int64_t n_tokens, int Hq, int Hkv, int d,
                float theta, hipStream_t s);
// one new token per sample: q embedded in place, k embedded into k_dst + b * kv_batch, v copied to v_dst + b * kv_batch
// (rows, nullable: sample b's row lies rows[b] cache rows further on)
int launch_rope_append(uint16_t* q, const uint16_t* k, const uint16_t* v, const int32_t* positions, int n_tokens,
                       int Hq, int Hkv, int d, float theta, uint16_t* k_dst, uint16_t* v_dst, int64_t kv_batch,
                       hipStream_t s, const int32_t* rows = nullptr);
int launch_silu_mul(const uint16_t* gate, const uint16_t* up, uint16_t* out, int64_t n_elems, hipStream_t s);

// ---- decoding step over the KV cache (decode.hip) ---------------------------
size_t decode_workspace_bytes(int B, int N, int Hq, int Hkv, int d);
// kv_batch: elements between two samples' caches (0: dense, N * Hkv * d); n_cached_samples (nullable, device
// [B]): sample b attends over its first n_cached_samples[b] + 1 <= N rows only
int launch_decode_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out, float* lse, int B,
                       int N, int Hq, int Hkv, int d, float scale, void* ws, hipStream_t s, int64_t kv_batch = 0,
                       DecodeParts* hand_over = nullptr, const int32_t* n_cached_samples = nullptr);

}  // namespace vitcop
