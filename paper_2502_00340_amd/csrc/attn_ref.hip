// Filtered attention backward, scalar-FMA version (Sec. 3.1, Eq. 3-4).
//
// This is the fp32 check-mode implementation; it also accepts bf16 storage
// (arithmetic is fp32 either way).  It is simple rather than fast: one block
// per (kept row, head).  The tuned bf16 path lives in attn_mfma.hip.
//
//   dQ:     for a kept query i, over ALL keys j at positions <= pos(i)
//           (kept or filtered: Eq. 3 part with kept keys + Eq. 4 with filtered keys)
//   dK/dV:  for a kept key j, over the kept queries i >= j of the same
//           sequence and the query heads sharing the KV head (Eq. 3);
//           rows of filtered tokens are never produced.
#include "common.h"

namespace cf {

__device__ __forceinline__ int seq_of_row(const int32_t* cu_kept, int B, int S, int j) {
    if (cu_kept == nullptr) return j / S;
    int b = 0;
    while (b + 1 < B && cu_kept[b + 1] <= j) ++b;
    return b;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_dq_ref_kernel(
    const T* __restrict__ q_kept, const T* __restrict__ k_full, const T* __restrict__ v_full,
    const float* __restrict__ lse_full, const T* __restrict__ do_kept, const float* __restrict__ Drow,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ cu_kept, int B, int S, int Hq,
    int Hkv, int d, float scale, int n_max, const int32_t* __restrict__ n_dev, T* __restrict__ dq_kept) {
    __shared__ float qs[256], dos[256], dss[256], red[256];
    const int j = blockIdx.x, h = blockIdx.y, g = h / (Hq / Hkv);
    if (j >= live_rows(n_max, n_dev)) return;
    const int tid = threadIdx.x;
    const int b = seq_of_row(cu_kept, B, S, j);
    const int row = idx ? idx[j] : j;
    const int pos = row - b * S;
    const int Nq = Hq * d, Nkv = Hkv * d;
    if (tid < d) {
        qs[tid] = to_f32<T>(q_kept[(int64_t)j * Nq + h * d + tid]);
        dos[tid] = to_f32<T>(do_kept[(int64_t)j * Nq + h * d + tid]);
    }
    const float lse = lse_full[((int64_t)b * Hq + h) * S + pos];
    const float Dj = Drow[(int64_t)j * Hq + h];
    const int parts = 256 / d;
    const int c = tid % d, part = tid / d;
    float acc = 0.f;
    __syncthreads();
    for (int c0 = 0; c0 <= pos; c0 += 256) {
        const int key = c0 + tid;
        float ds = 0.f;
        if (key <= pos) {
            const T* kr = k_full + ((int64_t)b * S + key) * Nkv + g * d;
            const T* vr = v_full + ((int64_t)b * S + key) * Nkv + g * d;
            float s = 0.f, dp = 0.f;
            for (int e = 0; e < d; ++e) {
                s += qs[e] * to_f32<T>(kr[e]);
                dp += dos[e] * to_f32<T>(vr[e]);
            }
            ds = __expf(scale * s - lse) * (dp - Dj);
        }
        dss[tid] = ds;
        __syncthreads();
        const int len = min(256, pos + 1 - c0);
        if (part < parts) {
            for (int kk = part; kk < len; kk += parts)
                acc += dss[kk] * to_f32<T>(k_full[((int64_t)b * S + c0 + kk) * Nkv + g * d + c]);
        }
        __syncthreads();
    }
    red[tid] = (part < parts) ? acc : 0.f;
    __syncthreads();
    if (tid < d) {
        float s = 0.f;
        for (int p = 0; p < parts; ++p) s += red[p * d + tid];
        dq_kept[(int64_t)j * Nq + h * d + tid] = from_f32<T>(s * scale);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void attn_dkv_ref_kernel(
    const T* __restrict__ q_kept, const T* __restrict__ k_full, const T* __restrict__ v_full,
    const float* __restrict__ lse_full, const T* __restrict__ do_kept, const float* __restrict__ Drow,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ cu_kept, int B, int S, int Hq,
    int Hkv, int d, float scale, int n_max, const int32_t* __restrict__ n_dev, T* __restrict__ dk_kept,
    T* __restrict__ dv_kept) {
    __shared__ float ks[256], vs[256], ps[256], dss[256], redk[256], redv[256];
    const int j = blockIdx.x, g = blockIdx.y, G = Hq / Hkv;
    const int tid = threadIdx.x;
    const int n_live = live_rows(n_max, n_dev);
    if (j >= n_live) return;
    const int b = seq_of_row(cu_kept, B, S, j);
    const int rowj = idx ? idx[j] : j;
    const int end = cu_kept ? min(cu_kept[b + 1], n_live) : (b + 1) * S;   // kept rows of this sequence end here
    const int Nq = Hq * d, Nkv = Hkv * d;
    if (tid < d) {
        ks[tid] = to_f32<T>(k_full[(int64_t)rowj * Nkv + g * d + tid]);
        vs[tid] = to_f32<T>(v_full[(int64_t)rowj * Nkv + g * d + tid]);
    }
    const int parts = 256 / d;
    const int c = tid % d, part = tid / d;
    float acck = 0.f, accv = 0.f;
    __syncthreads();
    for (int hh = 0; hh < G; ++hh) {
        const int h = g * G + hh;
        for (int c0 = j; c0 < end; c0 += 256) {
            const int i = c0 + tid;
            float p = 0.f, ds = 0.f;
            if (i < end) {
                const int posi = (idx ? idx[i] : i) - b * S;
                const T* qr = q_kept + (int64_t)i * Nq + h * d;
                const T* dor = do_kept + (int64_t)i * Nq + h * d;
                float s = 0.f, dp = 0.f;
                for (int e = 0; e < d; ++e) {
                    s += to_f32<T>(qr[e]) * ks[e];
                    dp += to_f32<T>(dor[e]) * vs[e];
                }
                p = __expf(scale * s - lse_full[((int64_t)b * Hq + h) * S + posi]);
                ds = p * (dp - Drow[(int64_t)i * Hq + h]);
            }
            ps[tid] = p;
            dss[tid] = ds;
            __syncthreads();
            const int len = min(256, end - c0);
            if (part < parts) {
                for (int ii = part; ii < len; ii += parts) {
                    accv += ps[ii] * to_f32<T>(do_kept[(int64_t)(c0 + ii) * Nq + h * d + c]);
                    acck += dss[ii] * to_f32<T>(q_kept[(int64_t)(c0 + ii) * Nq + h * d + c]);
                }
            }
            __syncthreads();
        }
    }
    redk[tid] = (part < parts) ? acck : 0.f;
    redv[tid] = (part < parts) ? accv : 0.f;
    __syncthreads();
    if (tid < d) {
        float sk = 0.f, sv = 0.f;
        for (int p = 0; p < parts; ++p) { sk += redk[p * d + tid]; sv += redv[p * d + tid]; }
        dk_kept[(int64_t)j * Nkv + g * d + tid] = from_f32<T>(sk * scale);
        dv_kept[(int64_t)j * Nkv + g * d + tid] = from_f32<T>(sv);
    }
}

template <typename T>
static hipError_t launch_ref_t(const cf_layer_desc& L, float scale, const void* q_kept,
                               const void* k_full, const void* v_full, const float* lse_full,
                               const void* do_kept, const float* Drow, const int32_t* idx,
                               const int32_t* cu_kept, RowCount rows, void* dq_kept, void* dk_kept,
                               void* dv_kept, hipStream_t st) {
    const int n_kept = rows.n;      // grids cover the upper bound of the row count
    attn_dq_ref_kernel<T><<<dim3(n_kept, L.Hq), 256, 0, st>>>(
        (const T*)q_kept, (const T*)k_full, (const T*)v_full, lse_full, (const T*)do_kept, Drow, idx,
        cu_kept, L.B, L.S, L.Hq, L.Hkv, L.d, scale, n_kept, rows.dev, (T*)dq_kept);
    attn_dkv_ref_kernel<T><<<dim3(n_kept, L.Hkv), 256, 0, st>>>(
        (const T*)q_kept, (const T*)k_full, (const T*)v_full, lse_full, (const T*)do_kept, Drow, idx,
        cu_kept, L.B, L.S, L.Hq, L.Hkv, L.d, scale, n_kept, rows.dev, (T*)dk_kept, (T*)dv_kept);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_ref(const cf_layer_desc& L, float scale, const void* q_kept,
                               const void* k_full, const void* v_full, const float* lse_full,
                               const void* do_kept, const float* Drow, const int32_t* idx,
                               const int32_t* cu_kept, RowCount rows, void* dq_kept, void* dk_kept,
                               void* dv_kept, hipStream_t st) {
    if (L.dtype == CF_F32)
        return launch_ref_t<float>(L, scale, q_kept, k_full, v_full, lse_full, do_kept, Drow, idx,
                                   cu_kept, rows, dq_kept, dk_kept, dv_kept, st);
    return launch_ref_t<bf16_t>(L, scale, q_kept, k_full, v_full, lse_full, do_kept, Drow, idx,
                                cu_kept, rows, dq_kept, dk_kept, dv_kept, st);
}

}  // namespace cf
