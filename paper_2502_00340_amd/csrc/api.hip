// C ABI: argument validation (host only, before any launch) and the layer
// orchestration.  See include/centrifuge.h for the contract of each call.
#include <math.h>

#include <algorithm>

#include "common.h"

namespace cf {
hipError_t launch_attn_bwd_ref(const cf_layer_desc& L, float scale, const void* q_kept,
                               const void* k_full, const void* v_full, const float* lse_full,
                               const void* do_kept, const float* Drow, const int32_t* idx,
                               const int32_t* cu_kept, RowCount rows, void* dq_kept, void* dk_kept,
                               void* dv_kept, hipStream_t st);
bool attn_mfma_supported(const cf_layer_desc& L);
size_t attn_mfma_partial_bytes(const cf_layer_desc& L, int n_kept);
hipError_t launch_attn_bwd_mfma(const cf_layer_desc& L, float scale, const void* q_kept,
                                const void* k_full, const void* v_full, const void* o_kept,
                                const float* lse_full, const void* do_kept, float* stat,
                                const int32_t* idx, const int32_t* cu_kept, RowCount rows, void* dq_kept,
                                void* dk_kept, void* dv_kept, float* partials, hipStream_t st,
                                const void* o_full = nullptr, const void* q_full = nullptr);
}  // namespace cf

using namespace cf;

namespace {

inline bool misaligned(const void* p, size_t a = 16) { return ((uintptr_t)p % a) != 0; }
inline hipStream_t as_stream(cf_stream s) { return reinterpret_cast<hipStream_t>(s); }

#define CF_HIP(expr)                                   \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) return CF_ERR_HIP;      \
    } while (0)

cf_status check_dtype(int dtype) {
    return (dtype == CF_BF16 || dtype == CF_F32) ? CF_OK : CF_ERR_DTYPE;
}

bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

// attention-relevant fields only
cf_status check_attn_desc(const cf_layer_desc* L) {
    if (!L) return CF_ERR_NULL;
    cf_status s = check_dtype(L->dtype);
    if (s != CF_OK) return s;
    if (L->B <= 0 || L->S <= 0 || L->Hq <= 0 || L->Hkv <= 0 || L->d <= 0) return CF_ERR_SHAPE;
    if ((int64_t)L->B * L->S > (int64_t)1 << 30) return CF_ERR_SHAPE;
    if (L->Hq % L->Hkv != 0) return CF_ERR_SHAPE;
    if (L->dtype == CF_BF16) {
        if (L->d % 8 != 0) return CF_ERR_SHAPE;
        if (L->d != 64 && L->d != 128) return CF_ERR_UNSUPPORTED;      // a valid head size this build has no kernel for
        // the matrix-core attention kernels address K, V (per sequence) and Q, dO (per sequence's kept
        // rows) with 32-bit byte offsets
        // (the loads run up to four 64-row steps past a sequence's end before the range check stops them)
        if (((int64_t)L->S + 256) * L->Hq * L->d * 2 >= ((int64_t)1 << 32)) return CF_ERR_UNSUPPORTED;
    } else {
        if (!pow2(L->d) || L->d < 4 || L->d > 256) return CF_ERR_SHAPE;
    }
    if (!(L->softmax_scale >= 0.f)) return CF_ERR_SHAPE;
    return CF_OK;
}

cf_status check_layer_desc(const cf_layer_desc* L) {
    cf_status s = check_attn_desc(L);
    if (s != CF_OK) return s;
    if (L->H <= 0 || L->F <= 0) return CF_ERR_SHAPE;
    const int mult = L->dtype == CF_BF16 ? 8 : 4;
    if (L->H % mult || L->F % mult) return CF_ERR_SHAPE;
    if (L->H > 256 * 8 * mult) return CF_ERR_SHAPE;     // row-norm kernels keep a row in registers
    if (!(L->rms_eps >= 0.f)) return CF_ERR_SHAPE;
    if (L->dtype == CF_BF16) {
        // the matrix-core GEMM addresses an operand or an output with 32-bit byte offsets whose upper
        // half means "out of range": every matrix of the layer has to stay below 2 GiB
        const int64_t rows = std::max<int64_t>((int64_t)L->B * L->S, std::max(L->F, L->H)) + 256;
        const int64_t cols = std::max<int64_t>(std::max(L->F, L->H), (int64_t)L->Hq * L->d);
        if (rows * cols * 2 >= ((int64_t)1 << 31)) return CF_ERR_UNSUPPORTED;
    }
    return CF_OK;
}

float eff_scale(const cf_layer_desc& L) {
    return L.softmax_scale > 0.f ? L.softmax_scale : 1.0f / sqrtf((float)L.d);
}

// row statistics: D per (row, head), and for the matrix-core path also the scaled LSE
size_t attn_drow_bytes(const cf_layer_desc& L, int n_kept) {
    return align_up((size_t)2 * (size_t)(n_kept > 0 ? n_kept : 1) * L.Hq * sizeof(float), 256);
}

// D row statistics followed by the per-head dK/dV partials of the matrix-core path
size_t attn_ws_total(const cf_layer_desc& L, int n_kept) {
    return attn_drow_bytes(L, n_kept) + attn_mfma_partial_bytes(L, n_kept);
}

// bump allocator over the caller's workspace
struct Carver {
    unsigned char* base;
    size_t off = 0;
    explicit Carver(void* p) : base(static_cast<unsigned char*>(p)) {}
    void* take(size_t bytes) {
        void* r = base ? base + off : nullptr;
        off += align_up(bytes ? bytes : 1, 256);
        return r;
    }
};

struct LayerWs {
    void* index_ws;
    int32_t *idx, *cu_kept, *n_kept_dev;
    void *dy_k, *bufF0, *bufF1, *bufF2, *bufHa, *bufHb, *dr, *a_k, *da, *q_k, *dq, *dk, *dv;
    void* attn_ws;
    float* dg_partial;
    size_t total;
};

LayerWs carve_layer(const cf_layer_desc& L, int max_kept, void* ws) {
    const size_t e = dtype_size(L.dtype);
    const size_t N = (size_t)(max_kept > 0 ? max_kept : 1);
    const size_t T = (size_t)L.B * L.S;
    const size_t Nq = (size_t)L.Hq * L.d, Nkv = (size_t)L.Hkv * L.d;
    Carver c(ws);
    LayerWs w;
    w.index_ws = c.take(index_ws_bytes((int64_t)T));
    w.idx = (int32_t*)c.take(T * 4);
    w.cu_kept = (int32_t*)c.take((size_t)(L.B + 1) * 4);
    w.n_kept_dev = (int32_t*)c.take(4);
    w.dy_k = c.take(N * L.H * e);
    w.bufF0 = c.take(N * L.F * e);
    w.bufF1 = c.take(N * L.F * e);
    w.bufF2 = c.take(N * L.F * e);
    w.bufHa = c.take(N * L.H * e);
    w.bufHb = c.take(N * L.H * e);
    w.dr = c.take(N * L.H * e);
    w.a_k = c.take(N * Nq * e);
    w.da = c.take(N * Nq * e);
    w.q_k = c.take(N * Nq * e);
    w.dq = c.take(N * Nq * e);
    w.dk = c.take(N * Nkv * e);
    w.dv = c.take(N * Nkv * e);
    w.attn_ws = c.take(attn_ws_total(L, (int)N));
    w.dg_partial = (float*)c.take((size_t)rmsnorm_bwd_blocks((int)N) * L.H * 4);
    w.total = c.off;
    return w;
}

// o_full / q_full (nullable): the attention output and the queries at full length; the row-statistics
// pass then copies their kept rows (through idx) into the writable buffers o_kept / q_kept.
cf_status attn_dispatch(const cf_layer_desc& L, const void* q_kept, const void* k_full,
                        const void* v_full, const void* o_kept, const float* lse_full,
                        const void* do_kept, const int32_t* idx, const int32_t* cu_kept, RowCount rows,
                        void* dq_kept, void* dk_kept, void* dv_kept, void* attn_ws, hipStream_t st,
                        const void* o_full = nullptr, const void* q_full = nullptr) {
    const int n_kept = rows.n;
    if (n_kept <= 0) return CF_OK;
    const float scale = eff_scale(L);
    float* Drow = static_cast<float*>(attn_ws);
    float* partials = reinterpret_cast<float*>(static_cast<unsigned char*>(attn_ws) + attn_drow_bytes(L, n_kept));
    if (attn_mfma_supported(L)) {
        CF_HIP(launch_attn_bwd_mfma(L, scale, q_kept, k_full, v_full, o_kept, lse_full, do_kept, Drow, idx,
                                    cu_kept, rows, dq_kept, dk_kept, dv_kept, partials, st, o_full, q_full));
    } else {
        CF_HIP(launch_attn_rowdot(L.dtype, do_kept, o_full ? o_full : o_kept, rows, L.Hq, L.d, Drow, st,
                                  o_full ? idx : nullptr, const_cast<void*>(o_kept), q_full,
                                  const_cast<void*>(q_kept)));
        CF_HIP(launch_attn_bwd_ref(L, scale, q_kept, k_full, v_full, lse_full, do_kept, Drow, idx,
                                   cu_kept, rows, dq_kept, dk_kept, dv_kept, st));
    }
    return CF_OK;
}

// Everything after the keep index is launched.  rows: the live rows (a host count, or a device count
// with its upper bound); idx == nullptr means the dense backward (row j is token j).
// dy: the upstream gradient, compact [rows,H] when dy_is_full == false; when dy_is_full it is the
// full-length [T,H] tensor and its kept rows are read through idx (by the first GEMM's A-tile loads
// and by the SwiGLU pass, which also leaves the compact copy in w.dy_k for the GEMM that contracts
// over the kept tokens).
cf_status layer_core(const cf_layer_desc& L, const cf_saved& sv, const cf_weights& W,
                     const void* dy, bool dy_is_full, const int32_t* idx,
                     const int32_t* cu_kept, RowCount rows, cf_grads& G, const LayerWs& w, hipStream_t st) {
    const int dt = L.dtype;
    const size_t e = dtype_size(dt);
    const int N = rows.n;
    const int32_t* nd = rows.dev;
    const int H = L.H, F = L.F, Nq = L.Hq * L.d, Nkv = L.Hkv * L.d;
    const int64_t T = (int64_t)L.B * L.S;
    // main-gradient mode: the nine parameter gradients are fp32 buffers that this call adds to
    const bool mg = G.main_grad != 0;
    auto dw_gemm = [&](const void* A, const void* B, void* C, int M, int Ncols) {
        GemmSeg s{A, B, N};
        return launch_gemm(dt, 1, &s, 1, C, M, Ncols, mg ? 1.f : 0.f, st, 1.f, nullptr, 0, mg, nd);
    };

    if (N == 0) {   // nothing kept (known to the host): every gradient is zero, dx has no rows
        if (mg) return CF_OK;
        void* outs[9] = {G.dwq, G.dwk, G.dwv, G.dwo, G.dwg, G.dwu, G.dwd, G.dg1, G.dg2};
        size_t sz[9] = {(size_t)H * Nq, (size_t)H * Nkv, (size_t)H * Nkv, (size_t)Nq * H,
                        (size_t)H * F, (size_t)H * F, (size_t)F * H, (size_t)H, (size_t)H};
        for (int i = 0; i < 9; ++i) CF_HIP(launch_fill_zero(outs[i], sz[i] * e, st));
        return CF_OK;
    }
    if (dy_is_full && !idx) return CF_ERR_NULL;

    // ---- SwiGLU FFN: y = r + act*Wd --------------------------------------------
    // d_act = dy * Wd^T first; one pass over it then yields d_gate, d_up and act (the SwiGLU
    // product, rebuilt for dWd), so gate and up are read once
    void* d_act = w.bufF1;
    {   // [N,F] = [N,H] x [F,H]^T
        GemmSeg s{dy, W.wd, H};
        CF_HIP(launch_gemm(dt, 0, &s, 1, d_act, N, F, 0.f, st, 1.f, nullptr, 0, false, nd,
                           dy_is_full ? idx : nullptr, dy_is_full ? T : 0));
    }
    void* d_gate = w.bufF1;   // in place over d_act
    void* d_up = w.bufF0;
    void* act = w.bufF2;
    const void* dy_rows = dy_is_full ? w.dy_k : dy;
    CF_HIP(launch_swiglu_bwd(dt, d_act, sv.gate, sv.up, idx, rows, F, d_gate, d_up, act, st,
                             dy_is_full ? dy : nullptr, H, dy_is_full ? w.dy_k : nullptr));
    CF_HIP(dw_gemm(act, dy_rows, G.dwd, F, H));     // dWd = act^T * dy           [F,H]

    void* dh2 = w.bufHb;
    {   // dh2 = d_gate*Wg^T + d_up*Wu^T   [N,H], contraction over F twice
        GemmSeg s[2] = {{d_gate, W.wg, F}, {d_up, W.wu, F}};
        CF_HIP(launch_gemm(dt, 0, s, 2, dh2, N, H, 0.f, st, 1.f, nullptr, 0, false, nd));
    }
    // dr = dy + rmsnorm_bwd(dh2; r, g2);  dg2.  The pass has r and its rstd in registers, so it also
    // writes h2 = rmsnorm(r)*g2, the operand of the two parameter-gradient products below (which is why
    // they come after it: no norm-recompute pass of its own).
    void* h2 = w.bufHa;
    CF_HIP(launch_rmsnorm_bwd(dt, dh2, sv.r, W.g2, idx, dy_rows, rows, H, L.rms_eps, w.dr, w.dg_partial,
                              G.dg2, st, mg, h2));
    {   // dWg, dWu = h2^T * d_gate, d_up: one launch (7 rounds of tiles instead of 2 x 3.5 at the 8B shape)
        const int Ng[2] = {F, F};
        if (gemm_tn_groups_supported(dt, N, 2, Ng)) {
            const void* Bg[2] = {d_gate, d_up};
            void* Cg[2] = {G.dwg, G.dwu};
            CF_HIP(launch_gemm_tn_groups(h2, N, H, 2, Bg, Cg, Ng, st, mg ? 1.f : 0.f, mg, nd));
        } else {
            CF_HIP(dw_gemm(h2, d_gate, G.dwg, H, F));
            CF_HIP(dw_gemm(h2, d_up, G.dwu, H, F));
        }
    }

    // ---- attention block: r = x + attn_out*Wo ------------------------------------
    {
        GemmSeg s2{w.dr, W.wo, H};                        // da = dr * Wo^T      [N,Nq]
        CF_HIP(launch_gemm(dt, 0, &s2, 1, w.da, N, Nq, 0.f, st, 1.f, nullptr, 0, false, nd));
    }
    // the attention backward's row-statistics pass reads attn_out and q through idx and leaves their
    // compact copies in w.a_k, w.q_k (no gather kernel)
    const void* a_rows = idx ? w.a_k : sv.attn_out;
    const void* q_rows = idx ? w.q_k : sv.q;
    cf_status as = attn_dispatch(L, q_rows, sv.k, sv.v, a_rows, sv.lse, w.da, idx, cu_kept, rows, w.dq,
                                 w.dk, w.dv, w.attn_ws, st, idx ? sv.attn_out : nullptr, idx ? sv.q : nullptr);
    if (as != CF_OK) return as;
    CF_HIP(dw_gemm(a_rows, w.dr, G.dwo, Nq, H));          // dWo = a^T * dr      [Nq,H]

    if (sv.rope_cos) {      // transposed rotation of dq and dk at the original positions of the kept rows
        CF_HIP(launch_rope_bwd(dt, w.dq, idx, rows, L.Hq, L.d, L.S, sv.rope_cos, sv.rope_sin, st));
        CF_HIP(launch_rope_bwd(dt, w.dk, idx, rows, L.Hkv, L.d, L.S, sv.rope_cos, sv.rope_sin, st));
    }
    void* dh1 = w.bufHb;
    {   // dh1 = dq*Wq^T + dk*Wk^T + dv*Wv^T
        GemmSeg s[3] = {{w.dq, W.wq, Nq}, {w.dk, W.wk, Nkv}, {w.dv, W.wv, Nkv}};
        CF_HIP(launch_gemm(dt, 0, s, 3, dh1, N, H, 0.f, st, 1.f, nullptr, 0, false, nd));
    }
    // dx = dr + rmsnorm_bwd(dh1; x, g1);  dg1; h1 = rmsnorm(x)*g1 on the way (see h2 above)
    void* h1 = w.bufHa;
    CF_HIP(launch_rmsnorm_bwd(dt, dh1, sv.x, W.g1, idx, w.dr, rows, H, L.rms_eps, G.dx, w.dg_partial,
                              G.dg1, st, mg, h1));
    {   // dWq, dWk, dWv = h1^T * dq, dk, dv: one launch when the column groups fall on tile boundaries
        const int Ng[3] = {Nq, Nkv, Nkv};
        if (gemm_tn_groups_supported(dt, N, 3, Ng)) {
            const void* Bg[3] = {w.dq, w.dk, w.dv};
            void* Cg[3] = {G.dwq, G.dwk, G.dwv};
            CF_HIP(launch_gemm_tn_groups(h1, N, H, 3, Bg, Cg, Ng, st, mg ? 1.f : 0.f, mg, nd));
        } else {
            CF_HIP(dw_gemm(h1, w.dq, G.dwq, H, Nq));
            CF_HIP(dw_gemm(h1, w.dk, G.dwk, H, Nkv));
            CF_HIP(dw_gemm(h1, w.dv, G.dwv, H, Nkv));
        }
    }
    return CF_OK;
}

// ---- LoRA-adapted layer: base weights and gains frozen, adapters on q, k, v, o ---------------
struct LoraWs {
    LayerWs base;
    void *a_t;                  // [rank, max(H, Nq)]  transposed adapter
    void *u;                    // [N, rank]           scale * X * a
    void *tq, *tk, *tv, *to;    // [N, rank]           scale * dY * b^T
    void *dg_scratch;           // [H]
    void *splitk;               // fp32 parts of the split-K adapter GEMMs
    size_t total;
};

// Upper bound of what a split-K launch uses: parts <= CUs / tiles and a part holds at most
// tiles * 128 * 128 floats, so 64 KB per CU; sized for 512 CUs.
constexpr size_t kSplitKBytes = (size_t)32 << 20;

LoraWs carve_lora(const cf_layer_desc& L, int rank, int max_kept, void* ws) {
    LoraWs w;
    w.base = carve_layer(L, max_kept, ws);
    const size_t e = dtype_size(L.dtype);
    const size_t N = (size_t)(max_kept > 0 ? max_kept : 1);
    const size_t Nq = (size_t)L.Hq * L.d;
    Carver c(ws);
    c.off = w.base.total;
    w.a_t = c.take((size_t)rank * (Nq > (size_t)L.H ? Nq : (size_t)L.H) * e);
    w.u = c.take(N * rank * e);
    w.tq = c.take(N * rank * e);
    w.tk = c.take(N * rank * e);
    w.tv = c.take(N * rank * e);
    w.to = c.take(N * rank * e);
    w.dg_scratch = c.take((size_t)L.H * e);
    w.splitk = c.take(kSplitKBytes);
    w.total = c.off;
    return w;
}

// One adapted projection with input rows x [N,in] and output gradient dy [N,out]:
// t = scale*dy*b^T (kept for the caller's dX GEMM), db = (scale*x*a)^T*dy, da = x^T*t.
cf_status lora_proj(int dt, const void* x, const void* dy, const void* a, const void* b, RowCount rows, int in,
                    int out, int rank, float scale, void* t, void* da, void* db, const LoraWs& w,
                    hipStream_t st) {
    const int N = rows.n;
    const int32_t* nd = rows.dev;
    {   // t [N,rank] = scale * dy [N,out] * b [rank,out]^T
        GemmSeg s{dy, b, out};
        CF_HIP(launch_gemm(dt, 0, &s, 1, t, N, rank, 0.f, st, scale, w.splitk, kSplitKBytes, false, nd));
    }
    CF_HIP(launch_transpose(dt, a, in, rank, w.a_t, st));
    {   // u [N,rank] = scale * x [N,in] * a_t [rank,in]^T
        GemmSeg s{x, w.a_t, in};
        CF_HIP(launch_gemm(dt, 0, &s, 1, w.u, N, rank, 0.f, st, scale, w.splitk, kSplitKBytes, false, nd));
    }
    {   // db [rank,out] = u^T * dy
        GemmSeg s{w.u, dy, N};
        CF_HIP(launch_gemm(dt, 1, &s, 1, db, rank, out, 0.f, st, 1.f, w.splitk, kSplitKBytes, false, nd));
    }
    {   // da [in,rank] = x^T * t
        GemmSeg s{x, t, N};
        CF_HIP(launch_gemm(dt, 1, &s, 1, da, in, rank, 0.f, st, 1.f, w.splitk, kSplitKBytes, false, nd));
    }
    return CF_OK;
}

cf_status layer_core_lora(const cf_layer_desc& L, const cf_saved& sv, const cf_weights& W,
                          const cf_lora& A, const void* dy_rows, const int32_t* idx,
                          const int32_t* cu_kept, RowCount rows, cf_lora_grads& G, const LoraWs& lw,
                          hipStream_t st) {
    const LayerWs& w = lw.base;
    const int dt = L.dtype;
    const size_t e = dtype_size(dt);
    const int H = L.H, F = L.F, Nq = L.Hq * L.d, Nkv = L.Hkv * L.d, R = A.rank;
    const int N = rows.n;                   // the live rows, or their upper bound when the count is on the device
    const int32_t* nd = rows.dev;
    if (N == 0) {
        void* outs[8] = {G.daq, G.dbq, G.dak, G.dbk, G.dav, G.dbv, G.dao, G.dbo};
        size_t sz[8] = {(size_t)H * R, (size_t)R * Nq, (size_t)H * R, (size_t)R * Nkv,
                        (size_t)H * R, (size_t)R * Nkv, (size_t)Nq * R, (size_t)R * H};
        for (int i = 0; i < 8; ++i) CF_HIP(launch_fill_zero(outs[i], sz[i] * e, st));
        return CF_OK;
    }
    const void* a_rows = sv.attn_out;
    const void* q_rows = sv.q;
    if (idx) {
        CF_HIP(launch_gather(sv.attn_out, (int64_t)Nq * e, idx, rows, w.a_k, st));
        CF_HIP(launch_gather(sv.q, (int64_t)Nq * e, idx, rows, w.q_k, st));
        a_rows = w.a_k;
        q_rows = w.q_k;
    }
    // ---- frozen SwiGLU FFN: only the input gradient
    void* d_act = w.bufF1;
    {
        GemmSeg s{dy_rows, W.wd, H};
        CF_HIP(launch_gemm(dt, 0, &s, 1, d_act, N, F, 0.f, st, 1.f, nullptr, 0, false, nd));
    }
    void* d_gate = w.bufF1;
    void* d_up = w.bufF0;
    CF_HIP(launch_swiglu_bwd(dt, d_act, sv.gate, sv.up, idx, rows, F, d_gate, d_up, nullptr, st));
    void* dh2 = w.bufHb;
    {
        GemmSeg s[2] = {{d_gate, W.wg, F}, {d_up, W.wu, F}};
        CF_HIP(launch_gemm(dt, 0, s, 2, dh2, N, H, 0.f, st, 1.f, nullptr, 0, false, nd));
    }
    CF_HIP(launch_rmsnorm_bwd(dt, dh2, sv.r, W.g2, idx, dy_rows, rows, H, L.rms_eps, w.dr, w.dg_partial,
                              lw.dg_scratch, st));
    // ---- adapted O projection: input a [N,Nq], output gradient dr [N,H]
    cf_status ps = lora_proj(dt, a_rows, w.dr, A.ao, A.bo, rows, Nq, H, R, A.scale, lw.to, G.dao, G.dbo, lw, st);
    if (ps != CF_OK) return ps;
    {   // da = dr*Wo^T + t_o*a_o^T
        GemmSeg s[2] = {{w.dr, W.wo, H}, {lw.to, A.ao, R}};
        CF_HIP(launch_gemm(dt, 0, s, 2, w.da, N, Nq, 0.f, st, 1.f, nullptr, 0, false, nd));
    }
    cf_status as = attn_dispatch(L, q_rows, sv.k, sv.v, a_rows, sv.lse, w.da, idx, cu_kept, rows, w.dq,
                                 w.dk, w.dv, w.attn_ws, st);
    if (as != CF_OK) return as;
    if (sv.rope_cos) {
        CF_HIP(launch_rope_bwd(dt, w.dq, idx, rows, L.Hq, L.d, L.S, sv.rope_cos, sv.rope_sin, st));
        CF_HIP(launch_rope_bwd(dt, w.dk, idx, rows, L.Hkv, L.d, L.S, sv.rope_cos, sv.rope_sin, st));
    }
    // ---- adapted Q, K, V projections: input h1 [N,H]
    void* h1 = w.bufHa;
    CF_HIP(launch_rmsnorm_fwd(dt, sv.x, W.g1, idx, rows, H, L.rms_eps, h1, st));
    ps = lora_proj(dt, h1, w.dq, A.aq, A.bq, rows, H, Nq, R, A.scale, lw.tq, G.daq, G.dbq, lw, st);
    if (ps != CF_OK) return ps;
    ps = lora_proj(dt, h1, w.dk, A.ak, A.bk, rows, H, Nkv, R, A.scale, lw.tk, G.dak, G.dbk, lw, st);
    if (ps != CF_OK) return ps;
    ps = lora_proj(dt, h1, w.dv, A.av, A.bv, rows, H, Nkv, R, A.scale, lw.tv, G.dav, G.dbv, lw, st);
    if (ps != CF_OK) return ps;
    void* dh1 = w.bufHb;
    {   // dh1 = dq*Wq^T + dk*Wk^T + dv*Wv^T, then += t_q*a_q^T + t_k*a_k^T + t_v*a_v^T
        GemmSeg s[3] = {{w.dq, W.wq, Nq}, {w.dk, W.wk, Nkv}, {w.dv, W.wv, Nkv}};
        CF_HIP(launch_gemm(dt, 0, s, 3, dh1, N, H, 0.f, st, 1.f, nullptr, 0, false, nd));
        GemmSeg s2[3] = {{lw.tq, A.aq, R}, {lw.tk, A.ak, R}, {lw.tv, A.av, R}};
        CF_HIP(launch_gemm(dt, 0, s2, 3, dh1, N, H, 1.f, st, 1.f, nullptr, 0, false, nd));
    }
    CF_HIP(launch_rmsnorm_bwd(dt, dh1, sv.x, W.g1, idx, w.dr, rows, H, L.rms_eps, G.dx, w.dg_partial,
                              lw.dg_scratch, st));
    return CF_OK;
}

cf_status check_layer_ptrs(const cf_saved* sv, const cf_weights* W, const void* dy, const cf_grads* G) {
    if (!sv || !W || !dy || !G) return CF_ERR_NULL;
    const void* req[] = {sv->x, sv->q, sv->k, sv->v, sv->attn_out, sv->lse, sv->r, sv->gate, sv->up,
                         W->wq, W->wk, W->wv, W->wo, W->wg, W->wu, W->wd, W->g1, W->g2,
                         G->dwq, G->dwk, G->dwv, G->dwo, G->dwg, G->dwu, G->dwd, G->dg1, G->dg2, G->dx,
                         dy};
    for (const void* p : req) {
        if (!p) return CF_ERR_NULL;
    }
    for (const void* p : req) {
        if (misaligned(p)) return CF_ERR_SHAPE;
    }
    if ((sv->rope_cos == nullptr) != (sv->rope_sin == nullptr)) return CF_ERR_NULL;
    if (sv->rope_cos && (misaligned(sv->rope_cos) || misaligned(sv->rope_sin))) return CF_ERR_SHAPE;
    if (G->main_grad != 0 && G->main_grad != 1) return CF_ERR_SHAPE;
    return CF_OK;
}

cf_status check_rope(const cf_layer_desc* L, const cf_saved* sv) {
    if (!sv->rope_cos) return CF_OK;
    const int vn = L->dtype == CF_BF16 ? 8 : 4;
    return (L->d % 2 == 0 && (L->d / 2) % vn == 0) ? CF_OK : CF_ERR_SHAPE;
}

}  // namespace

extern "C" {

const char* cf_status_str(cf_status s) {
    switch (s) {
        case CF_OK: return "ok";
        case CF_ERR_NULL: return "required pointer is NULL";
        case CF_ERR_SHAPE: return "invalid, misaligned or inconsistent size";
        case CF_ERR_DTYPE: return "unknown dtype";
        case CF_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case CF_ERR_UNSUPPORTED: return "not supported by this build";
        case CF_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char* cf_version(void) { return "centrifuge-mi355x 0.1 (gfx950)"; }

size_t cf_index_workspace_bytes(int64_t n_tokens) { return index_ws_bytes(n_tokens); }

cf_status cf_build_keep_index(const uint8_t* mask, int32_t B, int32_t S, int32_t* idx,
                              int32_t* cu_kept, int32_t* n_kept_dev, int32_t* n_kept_host, void* ws,
                              size_t ws_bytes, cf_stream stream) {
    if (!mask || !idx || !cu_kept) return CF_ERR_NULL;
    if (B <= 0 || S <= 0 || (int64_t)B * S > ((int64_t)1 << 30)) return CF_ERR_SHAPE;
    if (misaligned(idx, 4) || misaligned(cu_kept, 4) || (n_kept_dev && misaligned(n_kept_dev, 4)))
        return CF_ERR_SHAPE;
    const size_t need = index_ws_bytes((int64_t)B * S);
    if (!ws || ws_bytes < need || misaligned(ws, 256)) return CF_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    CF_HIP(launch_keep_index(mask, B, S, idx, cu_kept, n_kept_dev, ws, st));
    if (n_kept_host) {
        CF_HIP(hipMemcpyAsync(n_kept_host, cu_kept + B, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        CF_HIP(hipStreamSynchronize(st));
    }
    return CF_OK;
}

cf_status cf_build_keep_index_static(const uint8_t* mask, int32_t B, int32_t S, int32_t* idx,
                                     int32_t* cu_kept, int32_t* n_kept_dev, cf_stream stream) {
    if (!mask || !idx || !cu_kept) return CF_ERR_NULL;
    if (B <= 0 || S <= 0 || (int64_t)B * S > ((int64_t)1 << 30)) return CF_ERR_SHAPE;
    if (misaligned(idx, 4) || misaligned(cu_kept, 4) || (n_kept_dev && misaligned(n_kept_dev, 4)))
        return CF_ERR_SHAPE;
    if ((int64_t)B * S > IDX_STATIC_MAX_TOKENS) return CF_ERR_UNSUPPORTED;    // beyond the built-in scratch
    CF_HIP(launch_keep_index_static(mask, B, S, idx, cu_kept, n_kept_dev, as_stream(stream)));
    return CF_OK;
}

cf_status cf_gather_rows(const void* src, int64_t src_rows, int64_t cols, int32_t dtype,
                         const int32_t* idx, const int32_t* n_kept_dev, int32_t max_kept, void* dst,
                         cf_stream stream) {
    if (!src || !idx || !dst) return CF_ERR_NULL;
    cf_status s = check_dtype(dtype);
    if (s != CF_OK) return s;
    if (src_rows <= 0 || cols <= 0 || max_kept < 0) return CF_ERR_SHAPE;
    const int64_t row_bytes = cols * (int64_t)dtype_size(dtype);
    if (row_bytes % 4 != 0 || misaligned(src, 4) || misaligned(dst, 4) || misaligned(idx, 4) ||
        (n_kept_dev && misaligned(n_kept_dev, 4)))
        return CF_ERR_SHAPE;
    if (row_bytes / 4 > INT32_MAX) return CF_ERR_SHAPE;
    CF_HIP(launch_gather(src, row_bytes, idx, RowCount{max_kept, n_kept_dev}, dst, as_stream(stream)));
    return CF_OK;
}

cf_status cf_linear_bwd_reduced(const void* x_kept, const void* dy_kept, const void* w, int32_t n_kept,
                                int32_t in, int32_t out, int32_t dtype, void* dx_kept, void* dw,
                                float dw_beta, cf_stream stream) {
    cf_status s = check_dtype(dtype);
    if (s != CF_OK) return s;
    if (!dy_kept) return CF_ERR_NULL;
    if (dx_kept && !w) return CF_ERR_NULL;
    if (dw && !x_kept) return CF_ERR_NULL;
    if (n_kept < 0 || in <= 0 || out <= 0) return CF_ERR_SHAPE;
    const int mult = dtype == CF_BF16 ? 8 : 4;
    if (in % mult || out % mult) return CF_ERR_SHAPE;
    if (dw_beta != 0.f && dw_beta != 1.f) return CF_ERR_SHAPE;
    if (dtype == CF_BF16) {     // 32-bit byte offsets with the upper half reserved (see check_layer_desc)
        const int64_t rows = std::max<int64_t>(n_kept, in) + 256, cols = std::max(in, out);
        if (rows * cols * 2 >= ((int64_t)1 << 31)) return CF_ERR_UNSUPPORTED;
    }
    if (misaligned(dy_kept) || (w && misaligned(w)) || (x_kept && misaligned(x_kept)) ||
        (dx_kept && misaligned(dx_kept)) || (dw && misaligned(dw)))
        return CF_ERR_SHAPE;
    hipStream_t st = as_stream(stream);
    if (dx_kept && n_kept > 0) {
        GemmSeg seg{dy_kept, w, out};
        CF_HIP(launch_gemm(dtype, 0, &seg, 1, dx_kept, n_kept, in, 0.f, st));
    }
    if (dw) {
        GemmSeg seg{x_kept, dy_kept, n_kept};
        CF_HIP(launch_gemm(dtype, 1, &seg, 1, dw, in, out, dw_beta, st));
    }
    return CF_OK;
}

size_t cf_attn_workspace_bytes(const cf_layer_desc* desc, int32_t n_kept) {
    if (check_attn_desc(desc) != CF_OK || n_kept < 0) return 0;
    return attn_ws_total(*desc, n_kept);
}

cf_status cf_attn_bwd_filtered(const cf_layer_desc* desc, const void* q_kept, const void* k_full,
                               const void* v_full, const void* o_kept, const float* lse_full,
                               const void* do_kept, const int32_t* idx, const int32_t* cu_kept,
                               int32_t n_kept, void* dq_kept, void* dk_kept, void* dv_kept, void* ws,
                               size_t ws_bytes, cf_stream stream) {
    cf_status s = check_attn_desc(desc);
    if (s != CF_OK) return s;
    const void* req[] = {q_kept, k_full, v_full, o_kept, lse_full, do_kept, idx, cu_kept,
                         dq_kept, dk_kept, dv_kept};
    for (const void* p : req) {
        if (!p) return CF_ERR_NULL;
    }
    if (n_kept < 0 || (int64_t)n_kept > (int64_t)desc->B * desc->S) return CF_ERR_SHAPE;
    const int mult = desc->dtype == CF_BF16 ? 8 : 4;
    if ((desc->Hq * desc->d) % mult || (desc->Hkv * desc->d) % mult) return CF_ERR_SHAPE;
    for (const void* p : req) {
        if (misaligned(p, (p == idx || p == cu_kept || p == lse_full) ? 4 : 16)) return CF_ERR_SHAPE;
    }
    if (!ws || misaligned(ws, 256) || ws_bytes < cf_attn_workspace_bytes(desc, n_kept))
        return CF_ERR_WORKSPACE;
    return attn_dispatch(*desc, q_kept, k_full, v_full, o_kept, lse_full, do_kept, idx, cu_kept,
                         RowCount{n_kept, nullptr}, dq_kept, dk_kept, dv_kept, ws, as_stream(stream));
}

size_t cf_layer_workspace_bytes(const cf_layer_desc* desc, int32_t max_kept) {
    if (check_layer_desc(desc) != CF_OK || max_kept < 0) return 0;
    return carve_layer(*desc, max_kept, nullptr).total;
}

cf_status cf_layer_bwd_filtered(const cf_layer_desc* desc, const cf_saved* saved, const cf_weights* w,
                                const void* dy_full, const uint8_t* mask, int32_t max_kept, cf_grads* grads,
                                int32_t* idx_out, int32_t* cu_kept_out, int32_t* n_kept_dev_out,
                                int32_t* n_kept_host, void* ws, size_t ws_bytes, cf_stream stream) {
    cf_status s = check_layer_desc(desc);
    if (s != CF_OK) return s;
    s = check_layer_ptrs(saved, w, dy_full, grads);
    if (s != CF_OK) return s;
    s = check_rope(desc, saved);
    if (s != CF_OK) return s;
    if (!mask) return CF_ERR_NULL;
    if ((idx_out && misaligned(idx_out, 4)) || (cu_kept_out && misaligned(cu_kept_out, 4)) ||
        (n_kept_dev_out && misaligned(n_kept_dev_out, 4)))
        return CF_ERR_SHAPE;
    const int T = desc->B * desc->S;
    if (max_kept < 0) return CF_ERR_SHAPE;
    if (max_kept == 0 || max_kept > T) max_kept = T;
    if (!ws || misaligned(ws, 256)) return CF_ERR_WORKSPACE;
    LayerWs wk = carve_layer(*desc, max_kept, ws);
    if (ws_bytes < wk.total) return CF_ERR_WORKSPACE;
    hipStream_t st = as_stream(stream);
    int32_t* idx = idx_out ? idx_out : wk.idx;
    int32_t* cu = cu_kept_out ? cu_kept_out : wk.cu_kept;
    int32_t* n_dev = n_kept_dev_out ? n_kept_dev_out : wk.n_kept_dev;
    CF_HIP(launch_keep_index(mask, desc->B, desc->S, idx, cu, n_dev, wk.index_ws, st));
    // the count stays on the device: every later kernel reads it there, nothing waits for the host
    s = layer_core(*desc, *saved, *w, dy_full, true, idx, cu, RowCount{max_kept, n_dev}, *grads, wk, st);
    if (s != CF_OK) return s;
    // The host's copy of the count is queued behind the layer's kernels: the caller can read it only
    // after synchronising with the stream anyway, and ahead of them the copy would sit in their way.
    if (n_kept_host)
        CF_HIP(hipMemcpyAsync(n_kept_host, n_dev, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    return CF_OK;
}

cf_status cf_layer_bwd_compact(const cf_layer_desc* desc, const cf_saved* saved, const cf_weights* w,
                               const void* dy_kept, const int32_t* idx, const int32_t* cu_kept,
                               int32_t n_kept, cf_grads* grads, void* ws, size_t ws_bytes,
                               cf_stream stream) {
    cf_status s = check_layer_desc(desc);
    if (s != CF_OK) return s;
    s = check_layer_ptrs(saved, w, dy_kept, grads);
    if (s != CF_OK) return s;
    s = check_rope(desc, saved);
    if (s != CF_OK) return s;
    if (!idx || !cu_kept) return CF_ERR_NULL;
    if (misaligned(idx, 4) || misaligned(cu_kept, 4)) return CF_ERR_SHAPE;
    const int T = desc->B * desc->S;
    if (n_kept < 0 || n_kept > T) return CF_ERR_SHAPE;
    if (!ws || misaligned(ws, 256)) return CF_ERR_WORKSPACE;
    LayerWs wk = carve_layer(*desc, n_kept, ws);
    if (ws_bytes < wk.total) return CF_ERR_WORKSPACE;
    return layer_core(*desc, *saved, *w, dy_kept, false, idx, cu_kept, RowCount{n_kept, nullptr}, *grads, wk,
                      as_stream(stream));
}

cf_status cf_layer_bwd_compact_dev(const cf_layer_desc* desc, const cf_saved* saved, const cf_weights* w,
                                   const void* dy_kept, const int32_t* idx, const int32_t* cu_kept,
                                   const int32_t* n_kept_dev, int32_t max_kept, cf_grads* grads, void* ws,
                                   size_t ws_bytes, cf_stream stream) {
    cf_status s = check_layer_desc(desc);
    if (s != CF_OK) return s;
    s = check_layer_ptrs(saved, w, dy_kept, grads);
    if (s != CF_OK) return s;
    s = check_rope(desc, saved);
    if (s != CF_OK) return s;
    if (!idx || !cu_kept || !n_kept_dev) return CF_ERR_NULL;
    if (misaligned(idx, 4) || misaligned(cu_kept, 4) || misaligned(n_kept_dev, 4)) return CF_ERR_SHAPE;
    const int T = desc->B * desc->S;
    if (max_kept < 0) return CF_ERR_SHAPE;
    if (max_kept == 0 || max_kept > T) max_kept = T;
    if (!ws || misaligned(ws, 256)) return CF_ERR_WORKSPACE;
    LayerWs wk = carve_layer(*desc, max_kept, ws);
    if (ws_bytes < wk.total) return CF_ERR_WORKSPACE;
    return layer_core(*desc, *saved, *w, dy_kept, false, idx, cu_kept, RowCount{max_kept, n_kept_dev}, *grads,
                      wk, as_stream(stream));
}

cf_status cf_layer_bwd_dense(const cf_layer_desc* desc, const cf_saved* saved, const cf_weights* w,
                             const void* dy_full, cf_grads* grads, void* ws, size_t ws_bytes,
                             cf_stream stream) {
    cf_status s = check_layer_desc(desc);
    if (s != CF_OK) return s;
    s = check_layer_ptrs(saved, w, dy_full, grads);
    if (s != CF_OK) return s;
    s = check_rope(desc, saved);
    if (s != CF_OK) return s;
    const int T = desc->B * desc->S;
    if (!ws || misaligned(ws, 256)) return CF_ERR_WORKSPACE;
    LayerWs wk = carve_layer(*desc, T, ws);
    if (ws_bytes < wk.total) return CF_ERR_WORKSPACE;
    return layer_core(*desc, *saved, *w, dy_full, false, nullptr, nullptr, RowCount{T, nullptr}, *grads, wk,
                      as_stream(stream));
}

size_t cf_lora_workspace_bytes(const cf_layer_desc* desc, int32_t rank, int32_t max_kept) {
    if (check_layer_desc(desc) != CF_OK || max_kept < 0 || rank <= 0) return 0;
    return carve_lora(*desc, rank, max_kept, nullptr).total;
}

cf_status cf_layer_bwd_lora(const cf_layer_desc* desc, const cf_saved* saved, const cf_weights* w,
                            const cf_lora* lora, const void* dy_full, const uint8_t* mask, int32_t max_kept,
                            cf_lora_grads* grads, int32_t* idx_out, int32_t* cu_kept_out,
                            int32_t* n_kept_dev_out, int32_t* n_kept_host, void* ws, size_t ws_bytes,
                            cf_stream stream) {
    cf_status s = check_layer_desc(desc);
    if (s != CF_OK) return s;
    if (!saved || !w || !lora || !dy_full || !grads) return CF_ERR_NULL;
    {
        const void* req[] = {saved->x, saved->q, saved->k, saved->v, saved->attn_out, saved->lse, saved->r,
                             saved->gate, saved->up, w->wq, w->wk, w->wv, w->wo, w->wg, w->wu, w->wd, w->g1,
                             w->g2, lora->aq, lora->bq, lora->ak, lora->bk, lora->av, lora->bv, lora->ao,
                             lora->bo, grads->daq, grads->dbq, grads->dak, grads->dbk, grads->dav,
                             grads->dbv, grads->dao, grads->dbo, grads->dx, dy_full};
        for (const void* p : req)
            if (!p) return CF_ERR_NULL;
        for (const void* p : req)
            if (misaligned(p)) return CF_ERR_SHAPE;
    }
    if ((saved->rope_cos == nullptr) != (saved->rope_sin == nullptr)) return CF_ERR_NULL;
    s = check_rope(desc, saved);
    if (s != CF_OK) return s;
    const int mult = desc->dtype == CF_BF16 ? 8 : 4;
    if (lora->rank <= 0 || lora->rank % mult || lora->rank > 1024) return CF_ERR_SHAPE;
    if (!(lora->scale == lora->scale)) return CF_ERR_SHAPE;
    if ((idx_out && misaligned(idx_out, 4)) || (cu_kept_out && misaligned(cu_kept_out, 4)) ||
        (n_kept_dev_out && misaligned(n_kept_dev_out, 4)))
        return CF_ERR_SHAPE;
    if (!ws || misaligned(ws, 256)) return CF_ERR_WORKSPACE;
    const int T = desc->B * desc->S;
    if (max_kept < 0) return CF_ERR_SHAPE;
    if (max_kept == 0 || max_kept > T) max_kept = T;
    hipStream_t st = as_stream(stream);
    if (!mask) {
        LoraWs lw = carve_lora(*desc, lora->rank, T, ws);
        if (ws_bytes < lw.total) return CF_ERR_WORKSPACE;
        if (n_kept_host) *n_kept_host = T;
        return layer_core_lora(*desc, *saved, *w, *lora, dy_full, nullptr, nullptr, RowCount{T, nullptr}, *grads,
                               lw, st);
    }
    LoraWs lw = carve_lora(*desc, lora->rank, max_kept, ws);
    if (ws_bytes < lw.total) return CF_ERR_WORKSPACE;
    int32_t* idx = idx_out ? idx_out : lw.base.idx;
    int32_t* cu = cu_kept_out ? cu_kept_out : lw.base.cu_kept;
    int32_t* n_dev = n_kept_dev_out ? n_kept_dev_out : lw.base.n_kept_dev;
    CF_HIP(launch_keep_index(mask, desc->B, desc->S, idx, cu, n_dev, lw.base.index_ws, st));
    // the count stays on the device, as in cf_layer_bwd_filtered: nothing here waits for the host
    const RowCount rows{max_kept, n_dev};
    CF_HIP(launch_gather(dy_full, (int64_t)desc->H * dtype_size(desc->dtype), idx, rows, lw.base.dy_k, st));
    s = layer_core_lora(*desc, *saved, *w, *lora, lw.base.dy_k, idx, cu, rows, *grads, lw, st);
    if (s != CF_OK) return s;
    if (n_kept_host)
        CF_HIP(hipMemcpyAsync(n_kept_host, n_dev, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    return CF_OK;
}

}  // extern "C"
