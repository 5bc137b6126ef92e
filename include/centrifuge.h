/*
 * centrifuge.h -- C ABI of the MI355X (gfx950) token-filtered decoder-layer backward.
 *
 * The library implements the hot path of backward token filtering with
 * activation filtering (paper Sec. 3): the upstream gradient of a layer is
 * row-sparse (filtered tokens carry zero gradient), so every per-token
 * operation runs on the kept rows only ("dimension-reduced dense GEMM",
 * Sec. 3.2), and the attention backward emits dK/dV for kept tokens only
 * while dQ of a kept query still sees every key/value (Sec. 3.1, Eq. 3-4),
 * which keeps the gradient handed to the layer below row-sparse.
 *
 * Conventions (all entry points)
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the
 *     library never allocates or frees device memory and keeps no state
 *     between calls.  Scratch space is the caller-provided workspace `ws`
 *     (256-byte aligned); its required size comes from the *_workspace_bytes
 *     calls.  Pointers named *_host are HOST pointers.
 *   - Tokens are flat rows t = b*S + s.  Matrices are row-major and dense
 *     (leading dimension = number of columns).  Weights are stored [in, out]
 *     (Y = X * W).  "kept"/compact tensors have one row per kept token in
 *     ascending token order.
 *   - Size limit in CF_BF16 mode: every matrix a call touches ([T,F], [F,H], ...) must stay
 *     below 2 GiB (the GEMM kernels use 32-bit byte offsets); larger requests return
 *     CF_ERR_UNSUPPORTED before anything is launched.
 *   - dtype CF_BF16: bfloat16 storage, fp32 accumulation and fp32 row
 *     statistics; CF_F32: fp32 everywhere (check mode, not tuned).  LSE is
 *     always fp32.  In CF_BF16 mode H, Hq*d, Hkv*d and F must be multiples of
 *     8 and d must be 64 or 128 (another multiple of 8 returns CF_ERR_UNSUPPORTED);
 *     in CF_F32 mode they must be multiples of 4 and d <= 256.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return without synchronising; the one exception
 *     (cf_build_keep_index with a host pointer) says so.
 *   - The number of kept tokens N_k is a DEVICE value after the index build.  Calls
 *     that take `n_kept_dev` + `max_kept` read it there: max_kept is the upper bound
 *     that buffers and launches are sized for, the kernels work on min(N_k, max_kept)
 *     rows, and nothing waits for the host.  Calls that take a plain `n_kept` are for
 *     callers that know the count (a fixed keep ratio, or after reading it back).
 *   - Errors: argument errors are detected on the host before anything is
 *     launched and reported as a cf_status; nothing is written in that case.
 *     A HIP runtime failure is reported as CF_ERR_HIP.
 */
#ifndef CENTRIFUGE_H
#define CENTRIFUGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CF_OK = 0,
    CF_ERR_NULL = 1,        /* a required pointer is NULL */
    CF_ERR_SHAPE = 2,       /* a size is non-positive, misaligned or inconsistent */
    CF_ERR_DTYPE = 3,       /* dtype enum out of range */
    CF_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or too small */
    CF_ERR_UNSUPPORTED = 5, /* valid request this build does not implement */
    CF_ERR_HIP = 6          /* HIP runtime error */
} cf_status;

typedef enum { CF_BF16 = 0, CF_F32 = 1 } cf_dtype;

typedef void* cf_stream;

/* Shape of one decoder layer (RMSNorm -> GQA causal attention -> residual ->
 * RMSNorm -> SwiGLU FFN -> residual) and of the batch. */
typedef struct {
    int32_t B, S;          /* sequences, tokens per sequence; T = B*S            */
    int32_t H;             /* hidden size                                        */
    int32_t Hq, Hkv, d;    /* query heads, key/value heads (Hq % Hkv == 0), head dim */
    int32_t F;             /* SwiGLU width                                       */
    int32_t dtype;         /* cf_dtype                                           */
    float rms_eps;         /* RMSNorm epsilon                                    */
    float softmax_scale;   /* 0 => 1/sqrt(d)                                     */
} cf_layer_desc;

/* Activations saved by the forward pass, full length (T rows). */
typedef struct {
    const void* x;         /* [T,H]     layer input                              */
    const void* q;         /* [T,Hq*d]  queries as used by attention             */
    const void* k;         /* [T,Hkv*d] keys                                     */
    const void* v;         /* [T,Hkv*d] values                                   */
    const void* attn_out;  /* [T,Hq*d]  attention output before the O projection */
    const float* lse;      /* [B,Hq,S]  log-sum-exp of the scaled causal scores  */
    const void* r;         /* [T,H]     x + attn_out*Wo (input of the 2nd norm)  */
    const void* gate;      /* [T,F]     rmsnorm2(r)*Wg                           */
    const void* up;        /* [T,F]     rmsnorm2(r)*Wu                           */
    /* Rotary position embedding of q and k (optional; both NULL = none).  The paper does not
     * mention it; the evaluated model families use it.  Tables [S, d/2] fp32 for position s and
     * frequency i; the forward rotated each head of the projected q and k as
     *   out[i] = x[i]*cos - x[i+d/2]*sin,  out[i+d/2] = x[i+d/2]*cos + x[i]*sin   (i < d/2),
     * q and k above are the rotated tensors, and the layer calls apply the transposed rotation
     * to dq and dk, at the ORIGINAL position of each kept row, before the projections' backward. */
    const float* rope_cos;
    const float* rope_sin;
} cf_saved;

typedef struct {
    const void *wq, *wk, *wv;  /* [H,Hq*d], [H,Hkv*d], [H,Hkv*d] */
    const void *wo;            /* [Hq*d,H] */
    const void *wg, *wu;       /* [H,F]    */
    const void *wd;            /* [F,H]    */
    const void *g1, *g2;       /* [H] RMSNorm gains */
} cf_weights;

/* Outputs.  Parameter gradients have the shapes of the parameters.  dx is [N_k,H]
 * compact for the filtered call and [T,H] for the dense call, always overwritten.
 *   main_grad == 0: parameter gradients in the storage dtype, overwritten.
 *   main_grad == 1: the nine parameter-gradient tensors are fp32 buffers (whatever the
 *     storage dtype) and the call ADDS this batch's gradient to them, without rounding
 *     the fp32 accumulators to the storage dtype first: gradient accumulation over
 *     micro-batches in a master-precision buffer.  With no kept token nothing is added. */
typedef struct {
    void *dwq, *dwk, *dwv, *dwo, *dwg, *dwu, *dwd, *dg1, *dg2;
    void *dx;
    int32_t main_grad;
} cf_grads;

const char* cf_status_str(cf_status s);

/* Library version string (static storage). */
const char* cf_version(void);

/* ---- A1: keep-index build (Sec. 3.2: shrink the sequence dimension) --------
 * Order-preserving compaction of the keep mask (Sec. 2.1 Eq. 2: 1 = token is
 * selected; any non-zero byte counts as kept).
 *   mask        [B*S] bytes, device
 *   idx         [>= number kept] int32, device: flat row of the j-th kept token, ascending
 *   cu_kept     [B+1] int32, device: kept tokens in sequences before b; cu_kept[B] = N_k
 *   n_kept_dev  [1] int32, device (nullable)
 *   n_kept_host [1] int32, host (nullable).  When non-NULL the call copies N_k
 *               back and synchronises the stream before returning.
 *   ws          device scratch of cf_index_workspace_bytes(B*S) bytes
 * idx must have room for B*S entries unless the caller knows N_k in advance. */
size_t cf_index_workspace_bytes(int64_t n_tokens);
cf_status cf_build_keep_index(const uint8_t* mask, int32_t B, int32_t S,
                              int32_t* idx, int32_t* cu_kept, int32_t* n_kept_dev,
                              int32_t* n_kept_host, void* ws, size_t ws_bytes, cf_stream stream);

/* The keep-index build for callers that cannot allocate device memory or carry a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  Same
 * arguments and results as cf_build_keep_index without the workspace and without the host copy:
 * the per-span counts (one per 8192 tokens) live in a device array built into the library (8 KiB per GPU, held until
 * the process ends), nothing is allocated, freed or copied to the host and the stream is not
 * synchronised.  At most 2^24 tokens (B*S); more returns CF_ERR_UNSUPPORTED before any launch.
 * All calls on one GPU share that array: calls that overlap on one GPU (two streams, two host
 * threads) race and must be serialised by the caller. */
cf_status cf_build_keep_index_static(const uint8_t* mask, int32_t B, int32_t S,
                                     int32_t* idx, int32_t* cu_kept, int32_t* n_kept_dev,
                                     cf_stream stream);

/* ---- A2: row gather (Sec. 3.2: remove the filtered rows of saved tensors) --
 * dst[j,:] = src[idx[j],:] for j < min(N_k, max_kept), N_k = *n_kept_dev (device; NULL: exactly
 * max_kept rows).  src is [src_rows, cols], dst has room for max_kept rows; cols*sizeof(elt) must be
 * a multiple of 4.  idx entries must lie in [0, src_rows) (not checked: they live on the device). */
cf_status cf_gather_rows(const void* src, int64_t src_rows, int64_t cols, int32_t dtype,
                         const int32_t* idx, const int32_t* n_kept_dev, int32_t max_kept, void* dst,
                         cf_stream stream);

/* ---- A3: dimension-reduced linear backward (Sec. 3.2, the two GEMM types) ---
 * For Y = X*W with W [in,out]:
 *   dx_kept [n_kept,in]  = dy_kept [n_kept,out] * W^T          (nullable: skipped)
 *   dw      [in,out]     = dw_beta*dw + x_kept^T [in,n_kept] * dy_kept   (nullable: skipped)
 * x_kept is [n_kept,in].  dw_beta is 0 (overwrite) or 1 (accumulate).
 * n_kept == 0 is valid: dw is zeroed (beta 0) or left alone (beta 1). */
cf_status cf_linear_bwd_reduced(const void* x_kept, const void* dy_kept, const void* w,
                                int32_t n_kept, int32_t in, int32_t out, int32_t dtype,
                                void* dx_kept, void* dw, float dw_beta, cf_stream stream);

/* ---- A5: filtered attention backward (Sec. 3.1, Eq. 3 and Eq. 4) -----------
 * Kept queries attend to ALL keys/values at positions <= their own (causal on
 * original positions) for dQ; dK and dV are produced for kept tokens only.
 *   q_kept, o_kept, do_kept  [n_kept,Hq*d]   compact rows (o = attention output, do = its gradient)
 *   k_full, v_full           [T,Hkv*d]       full length
 *   lse_full                 [B,Hq,S] fp32   forward's log-sum-exp over the full causal row
 *   idx [n_kept], cu_kept [B+1]              from cf_build_keep_index
 *   dq_kept [n_kept,Hq*d], dk_kept, dv_kept [n_kept,Hkv*d]   outputs, overwritten
 * dk/dv are summed over the Hq/Hkv query heads that share a key/value head.
 * Uses only B,S,Hq,Hkv,d,dtype,softmax_scale of desc. */
size_t cf_attn_workspace_bytes(const cf_layer_desc* desc, int32_t n_kept);
cf_status cf_attn_bwd_filtered(const cf_layer_desc* desc, const void* q_kept, const void* k_full,
                               const void* v_full, const void* o_kept, const float* lse_full,
                               const void* do_kept, const int32_t* idx, const int32_t* cu_kept,
                               int32_t n_kept, void* dq_kept, void* dk_kept, void* dv_kept,
                               void* ws, size_t ws_bytes, cf_stream stream);

/* ---- whole layer -----------------------------------------------------------
 * cf_layer_bwd_filtered: mask -> keep index -> all reduced GEMMs, row-local backward ops (SwiGLU,
 * RMSNorm, residuals; Sec. 3.2 "G (.) g") and the filtered attention backward.  No tensor is gathered
 * by a kernel of its own: the kept rows of dy_full, gate, up, r, x are read through the index by the
 * kernels that consume them, and those of attn_out and q are copied by the attention backward's
 * row-statistics pass.  dy_full is the upstream gradient on all T rows (rows of filtered tokens are
 * ignored).  Outputs: grads->dx compact [N_k,H] (the row-sparse gradient for the layer below), all
 * parameter gradients; idx_out [T] / cu_kept_out [B+1] / n_kept_dev_out [1] (device, each nullable)
 * receive the keep index and N_k; n_kept_host (HOST, nullable; page-locked memory keeps the copy
 * asynchronous) receives N_k through a copy queued behind the call's kernels: read it after
 * synchronising with the stream.
 * The call itself never synchronises: every kernel reads N_k on the device.
 *   max_kept: upper bound of N_k that the workspace and grads->dx are sized for; 0 or a value above
 *   T means T, which is always sufficient.  A caller that knows its keep ratio saves workspace.  If
 *   the mask keeps more than max_kept tokens the call processes the first max_kept kept tokens only
 *   and the result is not the layer's gradient: compare the N_k read back with max_kept.
 * cf_layer_bwd_dense: the same kernels with every token kept and no index; dx is [T,H].
 * cf_layer_bwd_compact: a layer BELOW the one whose call built the keep index
 * (Sec. 3.2: once the first gradient is reduced, every later gradient is; Sec. 3.1:
 * the sparsity is handed on to all front layers).  dy_kept [n_kept,H] is the compact
 * dx of the layer above; idx [n_kept] and cu_kept [B+1] (device) are the index that
 * call returned and n_kept its N_k.  Saved activations are still full length.
 * Outputs as for the filtered call.  Nothing is copied to the host and the stream is
 * not synchronised.
 * cf_layer_bwd_compact_dev: the same for a caller that has not read N_k back: n_kept_dev is the
 * device count the filtered call returned and max_kept the bound it was given, so a whole stack of
 * layers runs without a single synchronisation.
 * ws must hold cf_layer_workspace_bytes(desc, max_kept) bytes (compact call: max_kept >= n_kept). */
size_t cf_layer_workspace_bytes(const cf_layer_desc* desc, int32_t max_kept);
cf_status cf_layer_bwd_filtered(const cf_layer_desc* desc, const cf_saved* saved,
                                const cf_weights* w, const void* dy_full, const uint8_t* mask,
                                int32_t max_kept, cf_grads* grads, int32_t* idx_out,
                                int32_t* cu_kept_out, int32_t* n_kept_dev_out, int32_t* n_kept_host,
                                void* ws, size_t ws_bytes, cf_stream stream);
cf_status cf_layer_bwd_compact(const cf_layer_desc* desc, const cf_saved* saved,
                               const cf_weights* w, const void* dy_kept, const int32_t* idx,
                               const int32_t* cu_kept, int32_t n_kept, cf_grads* grads,
                               void* ws, size_t ws_bytes, cf_stream stream);
cf_status cf_layer_bwd_compact_dev(const cf_layer_desc* desc, const cf_saved* saved,
                                   const cf_weights* w, const void* dy_kept, const int32_t* idx,
                                   const int32_t* cu_kept, const int32_t* n_kept_dev, int32_t max_kept,
                                   cf_grads* grads, void* ws, size_t ws_bytes, cf_stream stream);
cf_status cf_layer_bwd_dense(const cf_layer_desc* desc, const cf_saved* saved,
                             const cf_weights* w, const void* dy_full, cf_grads* grads,
                             void* ws, size_t ws_bytes, cf_stream stream);

/* ---- low-rank adapters (Sec. 5.3: LoRA, rank 64, on the q, k, v and o projections) --------
 * The adapted projection is Y = X*W + scale * (X*a)*b with a [in, rank], b [rank, out]; the base
 * weights and the RMSNorm gains are frozen, so the call produces no gradient for them: every
 * linear layer only hands its input gradient on (reduced GEMM dX), and the adapters get
 *   da = scale * X_kept^T * (dY_kept * b^T),   db = scale * (X_kept * a)^T * dY_kept,
 * with dX_kept = dY_kept*W^T + scale * (dY_kept*b^T)*a^T.  Saved q, k, v, attn_out, r are the
 * tensors of the adapted forward.  rank must be a multiple of 8 (CF_BF16) or 4 (CF_F32). */
typedef struct {
    const void *aq, *bq;   /* [H,rank],    [rank,Hq*d]  */
    const void *ak, *bk;   /* [H,rank],    [rank,Hkv*d] */
    const void *av, *bv;   /* [H,rank],    [rank,Hkv*d] */
    const void *ao, *bo;   /* [Hq*d,rank], [rank,H]     */
    int32_t rank;
    float scale;           /* usually lora_alpha / rank */
} cf_lora;

/* Adapter gradients have the shapes of the adapters and are overwritten; dx is compact
 * [N_k,H] (or [T,H] when every token is kept because mask is NULL). */
typedef struct {
    void *daq, *dbq, *dak, *dbk, *dav, *dbv, *dao, *dbo;
    void *dx;
} cf_lora_grads;

/* cf_layer_bwd_lora: the filtered layer backward of a LoRA-adapted layer.  Arguments as for
 * cf_layer_bwd_filtered (max_kept, idx_out, cu_kept_out, n_kept_dev_out, n_kept_host included): the kept
 * count stays on the device, every kernel reads it there, and the call never synchronises (the split-K
 * launches of the rank-r products are planned for max_kept; a part of the contraction that lies past the
 * live count contributes zeros).  mask == NULL means "every token kept" (no index, no gather: the dense
 * LoRA backward of the same library; *n_kept_host, when given, is set to T at once).
 * ws must hold cf_lora_workspace_bytes(desc, rank, max_kept) bytes (max_kept 0 or above T means T). */
size_t cf_lora_workspace_bytes(const cf_layer_desc* desc, int32_t rank, int32_t max_kept);
cf_status cf_layer_bwd_lora(const cf_layer_desc* desc, const cf_saved* saved, const cf_weights* w,
                            const cf_lora* lora, const void* dy_full, const uint8_t* mask, int32_t max_kept,
                            cf_lora_grads* grads, int32_t* idx_out, int32_t* cu_kept_out,
                            int32_t* n_kept_dev_out, int32_t* n_kept_host, void* ws, size_t ws_bytes,
                            cf_stream stream);

/* ---- measurement probes (for the rooflines of Sec. 3.2's GEMMs and of the gather / row-local
 * kernels; not part of the method) ------------------------------------------------------------
 * cf_probe_mfma_bf16: n_blocks blocks of four waves; every wave runs `iters` passes over an 8 x 8
 *   grid of 16x16x32 bf16 MFMA accumulators (the GEMM kernels' wave tile) with all operands in
 *   registers and pseudo-random non-zero operand values: no LDS, no global traffic.  sink: device,
 *   n_blocks*256 floats, overwritten (keeps the work alive).  *flops_out (host, nullable) receives
 *   the flop count of the launch.  Timing it gives the matrix cores' sustained rate on this chip
 *   under its power limit: the measured ceiling that the GEMM kernels are compared with.
 * cf_probe_mfma_lds_bf16: the same loop with LDS fragment reads mixed in at the GEMM kernels' ratio
 *   and nothing waiting for them inside the loop: reads = 0 none, 1 = 16 16-byte reads per 64 MFMAs
 *   (the NT kernel's), 2 = 32 transposing 8-byte reads per 64 MFMAs (the TN kernel's).  Same arguments
 *   and flop count as cf_probe_mfma_bf16; reads outside 0..2 -> CF_ERR_SHAPE.  Shows what the reads
 *   alone cost next to the MFMAs (issue slots, power), apart from the operand stream that feeds them.
 * cf_probe_copy: dst[0..bytes) = src[0..bytes) (device pointers, 16-byte aligned, bytes % 16 == 0,
 *   no overlap): a plain streaming copy, the measured HBM ceiling (bytes read + bytes written per
 *   second) for the bandwidth-bound kernels, and the reference that scales profiler byte counters. */
cf_status cf_probe_mfma_bf16(int32_t n_blocks, int32_t iters, float* sink, double* flops_out,
                             cf_stream stream);
cf_status cf_probe_mfma_lds_bf16(int32_t n_blocks, int32_t iters, int32_t reads, float* sink,
                                 double* flops_out, cf_stream stream);
cf_status cf_probe_copy(const void* src, void* dst, size_t bytes, cf_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CENTRIFUGE_H */
