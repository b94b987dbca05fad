/*
 * libvitcop — MI355X (gfx950) kernels for the pruned-prefill hot path of ViTCoP
 * (arXiv 2601.17818): the [CLS]-attention filter over vision-encoder tokens
 * (Sec. 3.1), K-vector-norm saliency with top-k selection (Sec. 3.2.2, Sec. 3.3),
 * compaction of the survivors, and causal attention over them.
 *
 * Conventions for every entry point
 *  - Plain C ABI.  bf16 tensors are passed as uint16_t bit patterns.
 *  - Every tensor pointer is a DEVICE pointer owned by the caller, 16-byte
 *    aligned unless stated otherwise, rows contiguous, token-major.
 *  - The library allocates no device memory and carries no data from one call to
 *    the next (the only thing it remembers is that a kernel's shared-memory limit
 *    has been raised, a once-per-process flag that any thread may set again).
 *    Scratch memory comes from the caller through `ws` / `ws_bytes`; the size
 *    needed is returned by the matching *_workspace_bytes query.  The contents
 *    of `ws` need not be initialised and are undefined afterwards.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue work on it and return without synchronising.
 *  - Return value: VITCOP_OK or a negative status.  All argument validation
 *    happens on the host before any HIP call, so invalid arguments are
 *    reported even on a machine without a GPU.  No exception crosses the ABI.
 *    vitcop_last_error() returns a thread-local description of the last failure.
 *  - Outputs are fully overwritten.  Inputs must be finite.
 */
#ifndef VITCOP_H
#define VITCOP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VITCOP_OK            0
#define VITCOP_EINVAL      (-1)  /* null/misaligned pointer, negative size, keep > n_vis, Hq % Hkv != 0 ... */
#define VITCOP_EUNSUPPORTED (-2) /* shape outside what the kernels are built for */
#define VITCOP_EWORKSPACE  (-3)  /* ws is NULL or smaller than *_workspace_bytes */
#define VITCOP_EHIP        (-4)  /* a HIP call or launch failed */

/* Largest candidate count the selection kernel ranks per sample. */
#define VITCOP_MAX_CANDIDATES 16384

/* flags of vitcop_knorm_select */
#define VITCOP_NORMS_PRECOMPUTED 1u /* `norms` is an input holding the scores to rank */
#define VITCOP_NORMS_SQUARED     2u /* with PRECOMPUTED: `norms` holds squared norms; it is
                                       overwritten with their square roots before ranking */

const char* vitcop_last_error(void);
int vitcop_version(void);

/* ------------------------------------------------------------------------
 * Stage I filter (Sec. 3.1, Eq. 1; Alg. 1 Stage I).
 * For each image b and head h, softmax over the N+1 keys of the logits
 * scale * <q_cls[b,h], k[b,i,h]>; the score of patch i (token i+1) is the
 * sum over heads of its softmax weight.  [CLS] (token 0) takes part in the
 * normalisation but is neither scored nor a candidate.  The `keep` highest
 * scores survive, ties going to the lower index.
 *   q_cls      [B,H,d]      bf16, query of the [CLS] token
 *   k          [B,N+1,H,d]  bf16, keys, [CLS] at token 0
 *   scale      softmax scale; 0 selects 1/sqrt(d)
 *   scores_out [B,N] fp32, may be NULL
 *   idx_out    [B,keep] int32, ascending patch indices in [0,N)
 * d in {64,128}; N <= VITCOP_MAX_CANDIDATES; 0 <= keep <= N.
 */
size_t vitcop_filter_visual_workspace_bytes(int B, int N, int H, int d);
int vitcop_filter_visual(const uint16_t* q_cls, const uint16_t* k,
                         int B, int N, int H, int d, int keep, float scale,
                         float* scores_out, int32_t* idx_out,
                         void* ws, size_t ws_bytes, void* stream);

/* The same call for callers that cannot allocate device memory or hand over a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): arguments, outputs and kernels are
 * those of vitcop_filter_visual, and the logits live in a scratch array inside the library's own device
 * image, VITCOP_FILTER_STATIC_MAX_BYTES per GPU, held until the process ends.  The call allocates nothing.
 * Limit: B * H * (N+1) * 4 bytes must fit the array, else VITCOP_EUNSUPPORTED (use vitcop_filter_visual).
 * Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race on it; calls on one stream are ordered and safe.  Nothing in it needs clearing: each call
 * writes every entry it later reads.  Other errors as vitcop_filter_visual, plus VITCOP_EHIP if the array's
 * device address cannot be obtained.
 */
#define VITCOP_FILTER_STATIC_MAX_BYTES (4u << 20)
int vitcop_filter_visual_static(const uint16_t* q_cls, const uint16_t* k,
                                int B, int N, int H, int d, int keep, float scale,
                                float* scores_out, int32_t* idx_out, void* stream);

/* ------------------------------------------------------------------------
 * K-norm saliency and selection (Sec. 3.2.2, Eq. 4; Alg. 1 Stage III; "a
 * smaller norm corresponds to higher importance", Sec. 2.2).
 * norm_i = sqrt(sum over the Hkv heads and d channels of K[b,i,h,c]^2) for the
 * visual tokens i in [vis_start, vis_start+n_vis).  The `keep` smallest norms
 * survive, ties going to the lower index.  The output list holds, ascending,
 * every text position plus the surviving visual positions.
 *   k              [B,T,Hkv,d] bf16; token rows k_row_stride elements apart,
 *                  samples k_batch_stride elements apart (so K may sit inside
 *                  a fused QKV buffer); strides are multiples of 8 elements.
 *                  May be NULL with VITCOP_NORMS_PRECOMPUTED.
 *   norms          [B,n_vis] fp32: output, or input when PRECOMPUTED
 *                  (with SQUARED it is replaced by its square root).
 *                  Ranking uses exactly the fp32 values left in `norms`.
 *   keep_idx_out   [B,T'] int32 positions in [0,T), T' = T - n_vis + keep
 * Hkv*d % 8 == 0; n_vis <= VITCOP_MAX_CANDIDATES; 0 <= keep <= n_vis.
 */
size_t vitcop_knorm_select_workspace_bytes(int B, int n_vis);
int vitcop_knorm_select(const uint16_t* k, int64_t k_row_stride, int64_t k_batch_stride,
                        int B, int T, int Hkv, int d, int vis_start, int n_vis, int keep,
                        float* norms, int32_t* keep_idx_out, unsigned flags,
                        void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Compaction: the token removal implied by TopK(V_current, ...) in Alg. 1.
 * dst[b,j,:] = src[b, idx[b,j], :] for up to 8 tensors in one launch.
 * Out of place only; dst is dense [B,T_out,row_bytes].  row_bytes and the
 * strides are multiples of 4; a multiple of 16 (with 16-byte aligned
 * pointers) takes the fast path.  Indices must lie in [0,T_in): this is the
 * caller's contract and is not checked on the device.
 */
typedef struct {
    const void* src;
    void*       dst;
    int64_t     row_bytes;
    int64_t     src_row_stride_bytes;
    int64_t     src_batch_stride_bytes;
} vitcop_gather_t;
#define VITCOP_MAX_GATHER 8
int vitcop_compact(const vitcop_gather_t* tensors /* host array */, int n_tensors,
                   const int32_t* idx /* [B,T_out] device */, int B, int T_in, int T_out,
                   void* stream);

/* ------------------------------------------------------------------------
 * Attention over the surviving tokens: exact softmax(scale Q K^T [+ causal]) V,
 * the computation a FlashAttention kernel performs (Sec. 1, Sec. 2.2; the
 * 4 N^2 d term of Eq. 7).  Causal order is the order of the rows given, which
 * is the original order because keep lists ascend.  Query head h reads KV head
 * h / (Hq/Hkv).  No positional encoding is applied.
 *   q [B,N,Hq,d], k,v [B,N,Hkv,d] bf16, dense
 *   out [B,N,Hq,d] bf16;  lse_out [B,Hq,N] fp32 natural-log-sum-exp, may be NULL
 *   scale 0 selects 1/sqrt(d);  causal 0 or 1
 * d in {64, 128}.
 */
size_t vitcop_prefill_attn_workspace_bytes(int B, int N, int Hq, int Hkv, int d);
int vitcop_prefill_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                        uint16_t* out, float* lse_out,
                        int B, int N, int Hq, int Hkv, int d, float scale, int causal,
                        void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Supporting step: linear projection with the K-norm as a side output
 * ("K vectors from the LLM's attention module", Sec. 3.2.2).
 *   y[m, n] = bf16( sum_k x[m,k] * w[n,k] (+ residual[m,n]) ), fp32 accumulate.
 *   x [M,K] bf16 rows x_row_stride elements apart; w [N,K] bf16 dense
 *   (out_features x in_features); y [M,N] bf16 rows y_row_stride apart.
 *   residual: NULL, or [M,N] bf16 with rows res_row_stride apart (added in fp32
 *   before rounding).
 *   sumsq_parts: NULL, or fp32 [P][M] with P = vitcop_project_sumsq_parts(N):
 *   part p holds, per row, the sum of squares of the ROUNDED outputs of a
 *   fixed group of columns; the P parts added in index order give
 *   sum_n y[m,n]^2, i.e. the squared K-norm of Eq. 4 without re-reading K.
 *   ws: NULL, or device scratch of ws_bytes >= vitcop_project_workspace_bytes(M,N,K)
 *   (16-byte aligned, contents undefined afterwards).  With few rows (M <= 256: the
 *   sequence after pruning) the weights are nearly all of the traffic; given the
 *   scratch, such a call streams W once through a split-K kernel whose fp32 partials
 *   live there and are added in a fixed order.  workspace_bytes is 0 where that path
 *   does not apply; without scratch, or with too little, the call uses the big tiles.
 * K % 32 == 0, N % 16 == 0, strides multiples of 8; each operand below 2^31 elements.
 */
int vitcop_project_sumsq_parts(int N);
size_t vitcop_project_workspace_bytes(int M, int N, int K);
int vitcop_project(const uint16_t* x, int64_t x_row_stride, const uint16_t* w,
                   uint16_t* y, int64_t y_row_stride,
                   const uint16_t* residual, int64_t res_row_stride,
                   int M, int N, int K, float* sumsq_parts,
                   void* ws, size_t ws_bytes, void* stream);

/* Selection from the projection's side output: adds the P parts in index
 * order, takes the square root, writes norms_out (may be NULL) and ranks as
 * vitcop_knorm_select does.  sumsq_parts is [P][part_stride]; the value of
 * sample b, visual token i is at index b*T + vis_start + i of each part.
 */
int vitcop_select_from_sumsq(const float* sumsq_parts, int n_parts, int64_t part_stride,
                             int B, int T, int vis_start, int n_vis, int keep,
                             float* norms_out, int32_t* keep_idx_out, void* stream);

/* ------------------------------------------------------------------------
 * One attention layer of the prefill with pruning on entry (body of the layer
 * loop of Alg. 1): K projection of all T tokens with the norm side output,
 * selection, compaction of hidden states and K, Q/V projection of survivors,
 * causal attention, output projection (+ residual).  keep == n_vis skips the
 * pruning steps and gives the vanilla layer it is compared with.
 * All weights are [out_features, in_features] bf16.
 */
typedef struct {
    int B, T, D, Hq, Hkv, d;
    int vis_start, n_vis, keep;
    int residual;                 /* 1: y = x_kept + attn_out W_o^T */
    const uint16_t* x;            /* [B,T,D] */
    const uint16_t *wq, *wk, *wv, *wo;
    uint16_t* y;                  /* [B,T',D], T' = T - n_vis + keep */
    int32_t*  keep_idx;           /* [B,T'] out (may be NULL when keep == n_vis) */
    float*    norms;              /* [B,n_vis] out, may be NULL */
    const int32_t* positions_in;  /* [B,T] original positions, may be NULL */
    int32_t*  positions_out;      /* [B,T'] gathered positions, may be NULL */
    /* profiling hook: hipEvent_t handles (as void*), each NULL or an event the caller created;
     * recorded on the stream right before and right after the K projection of all tokens */
    void* ev_kproj_begin;
    void* ev_kproj_end;
} vitcop_layer_t;
size_t vitcop_layer_workspace_bytes(const vitcop_layer_t* L);
int vitcop_layer_prefill(const vitcop_layer_t* L, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Step-wise schedule (Alg. 1 layer loop, Eq. 8): runs n_layers attention
 * layers on one batch, pruning on entry to layer prune_layer[s] (0-indexed)
 * down to prune_keep[s] visual tokens using that layer's own K.
 * Weights of layer l: wq[l], wk[l], wv[l], wo[l] (host arrays of device
 * pointers).  h <- h + attention block output; no MLP, no normalisation.
 *   x [B,T,D] in;  y_out [B,T_final,D];  positions_out [B,T_final] (may be NULL)
 */
typedef struct {
    int B, T, D, Hq, Hkv, d, vis_start, n_vis;
    int n_layers, n_stages;
    const int* prune_layer;       /* host, ascending */
    const int* prune_keep;        /* host, non-increasing, <= n_vis */
    const uint16_t* x;
    const uint16_t* const* wq;    /* host arrays, n_layers device pointers each */
    const uint16_t* const* wk;
    const uint16_t* const* wv;
    const uint16_t* const* wo;
    uint16_t* y_out;
    int32_t*  positions_out;
} vitcop_schedule_t;
size_t vitcop_schedule_workspace_bytes(const vitcop_schedule_t* S);
int vitcop_schedule_prefill(const vitcop_schedule_t* S, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Visual Information Clustering (Sec. 3.2.1, Eq. 2-3; Alg. 2): density-peak
 * clustering of the visual tokens that survived Stage I, under a spatial
 * neighbourhood constraint.  Per image, with D_feat[i,j] = ||f_i - f_j||_2 and
 * D_spatial[i,j] = ||p_i - p_j||_2:
 *   rho_i   = sum_{j != i} exp(-(D_feat[i,j] / d_c)^2)                      (Eq. 2)
 *   delta_i = min D_feat[i,j] over j with rho_j > rho_i and D_spatial[i,j] <= tau,
 *             N_i the first such j reaching it (lower index on ties);
 *             none: delta_i = +inf, N_i = -1                                (Eq. 3)
 *   gamma_i = rho_i * delta_i (+inf when delta_i is); the n_centers highest gamma
 *             are centres (lower index on ties)
 *   labels: a token follows its parents N_i until it reaches a root, i.e. a centre
 *             or a token without parent; clusters are numbered 0..R-1 by the token
 *             index of their root (Alg. 2 Step 4 gives the same partition; a
 *             non-centre without parent, which the listing leaves undefined, is
 *             the root of its own cluster, so R >= n_centers).
 * All comparisons are made on the fp32 values written to rho_out / delta_out /
 * dist_out, so the labels are a deterministic function of those arrays.
 *   feats  [B,n,D] bf16, rows feat_row_stride elements apart, images
 *          feat_batch_stride apart (multiples of 8); D % 32 == 0
 *   pos    [B,n,2] fp32 positions (the paper's tau = 0.6 assumes coordinates
 *          normalised to the unit square)
 *   n_centers = ceil(n * alpha) is the caller's choice (alpha is not published)
 *   labels_out [B,n] int32;  n_clusters_out [B] int32 (= R)
 *   rho_out, delta_out [B,n] fp32, parent_out [B,n] int32: optional (NULL)
 *   dist_out: optional [B,n,n4] fp32 with n4 = n rounded up to a multiple of 4
 *          (row stride n4, pad undefined), receives D_feat with a zero diagonal
 * n <= VITCOP_VIC_MAX_TOKENS.  One image's features must stay below 2^31 elements.
 */
#define VITCOP_VIC_MAX_TOKENS 8192
size_t vitcop_vic_cluster_workspace_bytes(int B, int n, int D);
int vitcop_vic_cluster(const uint16_t* feats, int64_t feat_row_stride, int64_t feat_batch_stride,
                       const float* pos, int B, int n, int D, float d_c, float tau, int n_centers,
                       int32_t* labels_out, int32_t* n_clusters_out, float* rho_out, float* delta_out,
                       int32_t* parent_out, float* dist_out, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Visual-textual collaborative pruning and merging (Sec. 3.2.3, Eq. 5-6; Alg. 3).
 * Per image, given the cluster label of every visual token (vitcop_vic_cluster),
 * the number of clusters N_c, the tokens' K-vector norms (Eq. 4) and a budget B:
 *   q_c = floor(|C_c| * max(0, B - N_c) / n)                                 (Eq. 5)
 *   the q_c tokens of cluster c with the smallest norm are kept as they are
 *   ("elites", lower index on equal norms); the other tokens of the cluster are
 *   replaced by their mean (fp32 sums in ascending token order, rounded to bf16) (Eq. 6)
 * Output rows: the elites in ascending token index, then one merged row per
 * cluster that has non-elites, in label order; n_out = sum q_c + #merged <= B
 * whenever B >= N_c (with B < N_c there are no elites and N_c merged rows).
 * The paper treats the output as a set and does not say which position a merged
 * token takes: out_index names, for an elite, its token, and for a merged row the
 * lowest-index token it absorbed.
 *   feats [B,n,D] bf16 (strides in elements, multiples of 8), D % 8 == 0
 *   labels [B,n] int32 in [0, n_clusters[b]): the caller's contract;
 *   n_clusters [B] int32 (device);  k_norms [B,n] fp32
 *   out_feats [B,n,D] bf16 and out_index [B,n] int32: rows [0, n_out[b]) are written
 *   n_out [B] int32;  assign_out [B,n] int32, optional (NULL): output row of every token
 * n <= VITCOP_VIC_MAX_TOKENS.
 */
size_t vitcop_collab_prune_merge_workspace_bytes(int B, int n);
int vitcop_collab_prune_merge(const uint16_t* feats, int64_t feat_row_stride, int64_t feat_batch_stride,
                              const int32_t* labels, const int32_t* n_clusters, const float* k_norms,
                              int B, int n, int D, int budget, uint16_t* out_feats, int32_t* out_index,
                              int32_t* n_out, int32_t* assign_out, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * A full decoder layer of the language model around the pruned prefill.  The
 * paper prunes inside the layers of LLaVA's LLaMA-family decoder (Sec. 4.1; the
 * layer loop of Alg. 1) without restating that architecture; these are its
 * published pieces: pre-norm RMSNorm, rotary position embedding (rotate-half
 * pairing: channel i < d/2 pairs with i + d/2, angle = position * theta^(-2i/d)),
 * grouped-query attention, SiLU-gated MLP, two residual adds.
 */

/* y[m,:] = x[m,:] / sqrt(mean(x[m,:]^2) + eps) * weight, fp32 arithmetic, bf16 in/out.
 * x, y [M,D] with row strides in elements (multiples of 8); D % 8 == 0. */
int vitcop_rmsnorm(const uint16_t* x, int64_t x_row_stride, const uint16_t* weight, float eps,
                   uint16_t* y, int64_t y_row_stride, int M, int D, void* stream);

/* Rotary embedding IN PLACE on q [B,N,Hq,d] and k [B,N,Hkv,d] (dense; either may be NULL) with
 * explicit positions [B,N] int32: survivors of pruning keep their original positions.
 * d % 16 == 0; theta > 1. */
int vitcop_rope(uint16_t* q, uint16_t* k, const int32_t* positions, int B, int N, int Hq, int Hkv,
                int d, float theta, void* stream);

/* out = silu(gate) * up element-wise; n_elems % 8 == 0, 16-byte aligned pointers. */
int vitcop_silu_mul(const uint16_t* gate, const uint16_t* up, uint16_t* out, int64_t n_elems, void* stream);

/* One decoder layer with pruning on entry (body of the layer loop of Alg. 1 on a full layer):
 *   a = RMSNorm(h) ; K = a Wk^T for all T tokens, with the K-norms of Eq. 4 as a side output
 *   (taken before the rotary embedding, which does not change them) ; keep list by the
 *   Stage III rule ; gather of h, a, K and the positions ; Q, V of the survivors ; rotary
 *   embedding of Q, K at the ORIGINAL positions ; causal attention ; h1 = h_kept + O Wo^T ;
 *   y = h1 + (silu(b Wg^T) * (b Wu^T)) Wd^T with b = RMSNorm(h1).
 * keep == n_vis gives the vanilla layer.  Weights are [out_features, in_features] bf16.
 * D % 32 == 0, F % 32 == 0, d in {64,128}.
 */
typedef struct {
    int B, T, D, Hq, Hkv, d, F;      /* F: width of the MLP */
    int vis_start, n_vis, keep;
    float eps, theta;                 /* RMSNorm epsilon; rotary base */
    const uint16_t* h;                /* [B,T,D] */
    const int32_t* positions;         /* [B,T] */
    const uint16_t *ln1, *ln2;        /* [D] */
    const uint16_t *wq, *wk, *wv, *wo, *wg, *wu, *wd;
    uint16_t* y;                      /* [B,T',D] */
    int32_t* keep_idx;                /* [B,T'] out, may be NULL */
    int32_t* positions_out;           /* [B,T'] out, may be NULL */
    float* norms;                     /* [B,n_vis] out, may be NULL */
    /* KV cache of the layer for later decoding steps, may be NULL: K (after the rotary embedding) and V
     * of the T' kept tokens go to rows [0,T') of each sample's [cache_capacity, Hkv, d] block */
    uint16_t* k_cache;
    uint16_t* v_cache;
    int cache_capacity;               /* rows per sample, >= T' */
    /* A right-padded batch, may be NULL (then every sample has n_vis visual tokens).  n_vis_samples [B]
     * int32 device: sample b holds n_vis_samples[b] <= n_vis visual tokens at [vis_start, vis_start +
     * n_vis_samples[b]), its remaining text follows them directly, and the last n_vis - n_vis_samples[b] of
     * its T rows are padding (any finite values; under the causal mask no real token attends to them).
     * Sample b then keeps min(keep, n_vis_samples[b]) visual tokens; its output is again right-padded to
     * T' = T - n_vis + keep rows (padding rows repeat the last input row), and n_vis_samples_out [B]
     * (may be NULL) receives the new counts.  Rows of `norms` past a sample's count are written as 0. */
    const int32_t* n_vis_samples;
    int32_t* n_vis_samples_out;
} vitcop_decoder_layer_t;
size_t vitcop_decoder_layer_workspace_bytes(const vitcop_decoder_layer_t* L);
int vitcop_decoder_layer_prefill(const vitcop_decoder_layer_t* L, void* ws, size_t ws_bytes, void* stream);

/* Whole-model prefill over full decoder layers (layer loop of Alg. 1, Eq. 8): n_layers decoder
 * layers on one batch, pruning on entry to layer prune_layer[s] (0-indexed) down to prune_keep[s]
 * visual tokens by that layer's own K-norms (the Stage III rule; the paper's own schedule prunes
 * at layers 2 and 22, Sec. 4.1).  Weights of layer l: ln1[l], ..., wd[l] (host arrays of device
 * pointers).  The hidden state is carried between layers in bf16.
 *   h [B,T,D] in, positions [B,T] in;  y_out [B,T_final,D];  positions_out [B,T_final] (may be NULL)
 */
typedef struct {
    int B, T, D, Hq, Hkv, d, F, vis_start, n_vis;
    int n_layers, n_stages;
    float eps, theta;
    const int* prune_layer;           /* host, ascending */
    const int* prune_keep;            /* host, non-increasing, <= n_vis */
    const uint16_t* h;
    const int32_t* positions;
    const uint16_t* const* ln1;       /* host arrays, n_layers device pointers each */
    const uint16_t* const* ln2;
    const uint16_t* const* wq;
    const uint16_t* const* wk;
    const uint16_t* const* wv;
    const uint16_t* const* wo;
    const uint16_t* const* wg;
    const uint16_t* const* wu;
    const uint16_t* const* wd;
    uint16_t* y_out;
    int32_t* positions_out;
    /* KV caches, may be NULL: host arrays of n_layers device pointers, each [B, cache_capacity, Hkv, d];
     * layer l fills the rows of the tokens it kept (a pruned prefill leaves shorter caches in later layers) */
    uint16_t* const* k_cache;
    uint16_t* const* v_cache;
    int cache_capacity;
    /* Record of the Stage III decisions, may be NULL: host arrays of n_stages device pointers (single entries
     * may be NULL too).  Stage s writes the fp32 K-norms its selection ranked, [B, visual tokens present on
     * entry to its layer], and its keep list, [B, tokens the layer keeps] int32 indices into the sequence
     * that entered the layer. */
    float* const* stage_norms;
    int32_t* const* stage_keep_idx;
} vitcop_decoder_schedule_t;
size_t vitcop_decoder_schedule_workspace_bytes(const vitcop_decoder_schedule_t* S);
int vitcop_decoder_schedule_prefill(const vitcop_decoder_schedule_t* S, void* ws, size_t ws_bytes, void* stream);

/* The paper's whole in-model procedure (Alg. 1) on a batch: the decoder layers of S; on entry to
 * layer stage2_layer the n_vis visual tokens of every sample are clustered (Alg. 2: vitcop_vic_cluster on
 * their hidden states and grid positions vis_xy) and replaced by the per-cluster elites and one merged
 * token per cluster (Alg. 3: vitcop_collab_prune_merge with budget stage2_budget and that layer's K-norms,
 * Eq. 4); the stages of S (all at layers after stage2_layer) then prune by the Stage III rule.  The number
 * of visual tokens Stage II leaves is data-dependent (<= stage2_budget when the budget is at least the
 * number of clusters) and differs between samples: the call reads the B counts back and therefore
 * SYNCHRONISES the stream once, and from there on the batch is RIGHT-PADDED to its longest sample (see
 * vitcop_decoder_layer_t.n_vis_samples): the real tokens of a sample are a prefix of its rows, so under the
 * causal mask padding changes no real token's result.  A Stage III budget above a sample's count keeps all
 * of that sample's tokens.  The new visual block holds the elites in token order, then the merged tokens
 * in cluster order; a merged token takes the position of the lowest-index token it absorbed; padding rows
 * hold zeros (position 0) after Stage II and copies of a row of the same sample after Stage III.
 *   S->y_out [B,T,D] and S->positions_out [B,T] (may be NULL) are sized for T rows per sample and written
 *   densely as [B,T_final,...]; sample b's real rows are the first T_final_samples[b] of its T_final.
 *   KV caches (S->k_cache, S->v_cache): layer l writes rows [0, padded length) of every sample, of which
 *   the first cache_len_samples[l*B + b] are real; decoding over them needs equal lengths per layer.
 *   vis_xy [B,n_vis,2] fp32 device;  T_final: host int;  n_stage2, T_final_samples: host arrays of B ints,
 *   cache_len_samples: host array of n_layers*B ints (the three may be NULL)
 *   labels [B,n_vis], norms [B,n_vis] fp32, out_index [B,n_vis] (row b: n_stage2[b] entries): device
 *   outputs of Stage II, may be NULL
 * D % 32 == 0, n_vis <= VITCOP_VIC_MAX_TOKENS.
 */
typedef struct {
    vitcop_decoder_schedule_t S;
    int stage2_layer, stage2_budget, n_centers;
    float d_c, tau;
    const float* vis_xy;
    int* T_final;
    int* n_stage2;
    int32_t* labels;
    float* norms;
    int32_t* out_index;
    int* T_final_samples;
    int* cache_len_samples;
} vitcop_full_schedule_t;
size_t vitcop_full_schedule_workspace_bytes(const vitcop_full_schedule_t* F);
int vitcop_full_schedule_prefill(const vitcop_full_schedule_t* F, void* ws, size_t ws_bytes, void* stream);

/* One decoding step of the whole model after a (pruned) prefill (what Table 5 times per generated token):
 * for the new token of every sample, n_layers decoder layers; layer l projects the token (K, Q, V in one
 * launch), applies the rotary embedding at positions[b], appends K and V to row n_cached[l] of its cache,
 * attends over the n_cached[l] + 1 cached keys (vitcop_decode_attn's kernels) and runs the output
 * projection and the gated MLP with their residual adds.  The caches of a pruned prefill are shorter in
 * the layers after a pruning point, hence one length per layer.
 *   h [B,D], positions [B];  y_out [B,D];  k_cache[l], v_cache[l] [B, cache_capacity, Hkv, d]
 *   n_cached: host [n_layers], each < cache_capacity
 * B <= 256; d in {64,128}; D a multiple of 64, F of 128.  One to four samples run through weight-streaming
 * matrix-vector kernels that carry the norms, the rotary embedding, the cache append, the activation and
 * the residual adds (6 launches per layer); more samples through the few-row matrix-core projections.
 * All pointers are device pointers except the descriptor's own arrays (n_cached and the per-layer pointer
 * tables), which are host memory read during the call.  The call enqueues on `stream` and returns; the
 * caller advances n_cached after each step.
 * Caches of different lengths within a batch (what vitcop_full_schedule_prefill leaves when Stage II kept
 * different numbers of tokens per sample): n_cached_samples, DEVICE int32 [n_layers, B], may be NULL; sample
 * b's cache in layer l then holds n_cached_samples[l*B + b] rows, its new K and V go to that row and it
 * attends over that many rows + 1; n_cached[l] (host) must be the largest of layer l's entries (it sizes the
 * launch and is checked against the capacity; an entry above it is clamped).  The caller advances both.
 * Errors: VITCOP_EINVAL (null pointer, sizes, a full cache), VITCOP_EUNSUPPORTED (shape limits),
 * VITCOP_EWORKSPACE, VITCOP_EHIP.
 */
typedef struct {
    int B, D, Hq, Hkv, d, F, n_layers, cache_capacity;
    float eps, theta;
    const int* n_cached;
    const uint16_t* h;
    const int32_t* positions;
    const uint16_t* const* ln1;
    const uint16_t* const* ln2;
    const uint16_t* const* wq;
    const uint16_t* const* wk;
    const uint16_t* const* wv;
    const uint16_t* const* wo;
    const uint16_t* const* wg;
    const uint16_t* const* wu;
    const uint16_t* const* wd;
    uint16_t* const* k_cache;
    uint16_t* const* v_cache;
    uint16_t* y_out;
    const int32_t* n_cached_samples;
} vitcop_decoder_decode_t;
size_t vitcop_decoder_decode_workspace_bytes(const vitcop_decoder_decode_t* S);
int vitcop_decoder_decode_step(const vitcop_decoder_decode_t* S, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * One decoding step over the KV cache a (pruned) prefill left behind: for the new
 * token of every sample, out = softmax(scale * K q) V over ALL N cached keys.  This
 * is the per-token cost that Table 5 reports after pruning: one pass over K and V
 * per layer, so it shrinks with the cache.  Query head h reads KV head h / (Hq/Hkv).
 *   q [B,Hq,d], k, v [B,N,Hkv,d] bf16 dense;  out [B,Hq,d] bf16
 *   lse_out [B,Hq] fp32 natural-log-sum-exp, may be NULL;  scale 0 selects 1/sqrt(d)
 * d in {64,128}; N >= 1.
 */
size_t vitcop_decode_attn_workspace_bytes(int B, int N, int Hq, int Hkv, int d);
int vitcop_decode_attn(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                       float* lse_out, int B, int N, int Hq, int Hkv, int d, float scale,
                       void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VITCOP_H */
