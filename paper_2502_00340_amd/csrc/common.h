// Internal helpers shared by the HIP translation units of the library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "centrifuge.h"

namespace cf {

typedef unsigned short bf16_t;   // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t h) {
    return __uint_as_float(((unsigned)h) << 16);
}

// round-to-nearest-even; inputs are finite in every use here
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// two fp32 -> packed bf16 pair (round-to-nearest-even in hardware: v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_hw;
    bf16x2_hw v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(unsigned, v);
}

// 16-byte vector access of VN elements, widened to fp32
template <typename T> struct Vec;

template <> struct Vec<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void load(const float* p, float (&o)[4]) {
        float4 v = *reinterpret_cast<const float4*>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    __device__ static __forceinline__ void store(float* p, const float (&i)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(i[0], i[1], i[2], i[3]);
    }
};

template <> struct Vec<bf16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void load(const bf16_t* p, float (&o)[8]) {
        uint4 v = *reinterpret_cast<const uint4*>(p);
        unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static __forceinline__ void store(bf16_t* p, const float (&i)[8]) {
        uint4 v;
        v.x = pack_bf16x2(i[0], i[1]);
        v.y = pack_bf16x2(i[2], i[3]);
        v.z = pack_bf16x2(i[4], i[5]);
        v.w = pack_bf16x2(i[6], i[7]);
        *reinterpret_cast<uint4*>(p) = v;
    }
};

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Raises a kernel's dynamic LDS limit once per device (the attribute belongs to the device's
// copy of the kernel); `done` holds one bit per device ordinal.  Safe from several host threads:
// a second thread at worst sets the attribute again.
static inline hipError_t allow_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
static inline size_t dtype_size(int dtype) { return dtype == CF_F32 ? 4 : 2; }

// Number of live rows of a launch (kept tokens).  dev == nullptr: exactly n, known to the host.
// Otherwise the count lives on the device (the index build earlier on the same stream wrote it) and
// n is only its upper bound: it sizes grids and buffer strides, and every kernel works on
// min(*dev, n) rows, so no launch has to wait for the host to learn the count.
struct RowCount {
    int n;
    const int32_t* dev;
};
__device__ __forceinline__ int live_rows(int n, const int32_t* dev) {
    if (dev == nullptr) return n;
    const int v = *dev;
    return v < 0 ? 0 : (v < n ? v : n);
}

// ---- internal launchers (one per translation unit) --------------------------

// index.hip
size_t index_ws_bytes(int64_t n_tokens);
hipError_t launch_keep_index(const uint8_t* mask, int B, int S, int32_t* idx, int32_t* cu_kept,
                             int32_t* n_kept_dev, void* ws, hipStream_t st);
// the same with the per-block counts in a device array of the library's own (no workspace, no
// allocation); at most IDX_STATIC_MAX_TOKENS tokens
static constexpr int64_t IDX_STATIC_MAX_TOKENS = (int64_t)1 << 24;
hipError_t launch_keep_index_static(const uint8_t* mask, int B, int S, int32_t* idx, int32_t* cu_kept,
                                    int32_t* n_kept_dev, hipStream_t st);
hipError_t launch_gather(const void* src, int64_t cols_bytes, const int32_t* idx, RowCount rows,
                         void* dst, hipStream_t st);

// rowlocal.hip
// act (nullable) also receives silu(gate)*up; d_gate may alias d_act.  copy_src (nullable, needs idx):
// a full-length [.., copy_cols] tensor whose kept rows the same launch copies to copy_dst
// [n_rows, copy_cols] (the compact upstream gradient that the parameter-gradient GEMM contracts over).
hipError_t launch_swiglu_bwd(int dtype, const void* d_act, const void* gate, const void* up,
                             const int32_t* idx, RowCount rows, int F, void* d_gate, void* d_up,
                             void* act, hipStream_t st, const void* copy_src = nullptr, int copy_cols = 0,
                             void* copy_dst = nullptr);
hipError_t launch_rmsnorm_fwd(int dtype, const void* x, const void* g, const int32_t* idx,
                              RowCount rows, int H, float eps, void* h, hipStream_t st);
// dx_out = res + rmsnorm_bwd(dh; x, g); dg_partial is [rmsnorm_bwd_blocks(n_rows), H] fp32 scratch.
// dg_acc_f32: dg_out is fp32 [H] and the gain gradient is added to it instead of written.
// h_out (nullable, [n_rows, H]): also receives the normalised rows rmsnorm(x)*g, as launch_rmsnorm_fwd
// would write them.
int rmsnorm_bwd_blocks(int n_rows);
hipError_t launch_rmsnorm_bwd(int dtype, const void* dh, const void* x, const void* g,
                              const int32_t* idx, const void* res, RowCount rows, int H, float eps,
                              void* dx_out, float* dg_partial, void* dg_out, hipStream_t st,
                              bool dg_acc_f32 = false, void* h_out = nullptr);
// g[j, h*d + i] (in place, [n_rows, heads*d]): transposed rotary rotation at position idx[j] % S
// (idx null: j % S); cos, sin are [S, d/2] fp32
hipError_t launch_rope_bwd(int dtype, void* g, const int32_t* idx, RowCount rows, int heads, int d, int S,
                           const float* cos, const float* sin, hipStream_t st);
// D[j,h] = sum_c da[j,h*d+c] * a[row,h*d+c], row = a_idx ? a_idx[j] : j; with a_idx the same launch also
// writes the compact copies a_out[j,:] = a[row,:] and (q_src non-null) q_out[j,:] = q_src[row,:]
hipError_t launch_attn_rowdot(int dtype, const void* da, const void* a, RowCount rows, int Hq, int d,
                              float* D, hipStream_t st, const int32_t* a_idx = nullptr, void* a_out = nullptr,
                              const void* q_src = nullptr, void* q_out = nullptr);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);
// dst [cols, rows] = src [rows, cols]^T  (small matrices: the low-rank adapters)
hipError_t launch_transpose(int dtype, const void* src, int rows, int cols, void* dst, hipStream_t st);

// gemm.hip
struct GemmSeg {
    const void* A;
    const void* B;
    int K;
};
// C[M,N] = beta*C + alpha * sum_seg op(A_seg)*op(B_seg); all matrices dense row-major.
//   mode 0 ("NT"): A_seg [M,K], B_seg [N,K]      (C = A * B^T)
//   mode 1 ("TN"): A_seg [K,M], B_seg [K,N]      (C = A^T * B)
// c_f32 (bf16 dtype only): C is an fp32 matrix (a main-gradient buffer) and the accumulators are
// added to beta*C without rounding to bf16.
// n_dev (nullable): the kept-token count on the device; then the kept-token dimension of the product
// (M in mode 0, the K of segment 0 in mode 1) is only an upper bound and the kernel uses
// min(*n_dev, bound).  a_idx (nullable, mode 0, segment 0): row m of A is row a_idx[m] of a longer
// matrix (the gather of the upstream gradient folded into the A-tile loads); a_rows = rows of that matrix.
// splitk_ws (device, splitk_bytes, 16-byte aligned, may be null): scratch that lets a bf16 product
// with one segment, few output tiles and a long K run as a split-K launch (fp32 parts summed in a
// fixed order by a second kernel).
hipError_t launch_gemm(int dtype, int mode, const GemmSeg* segs, int nseg, void* C, int M, int N,
                       float beta, hipStream_t st, float alpha = 1.0f, void* splitk_ws = nullptr,
                       size_t splitk_bytes = 0, bool c_f32 = false, const int32_t* n_dev = nullptr,
                       const int32_t* a_idx = nullptr, int64_t a_rows = 0);

// One TN launch for up to three products that share A [K,M]: C_j [M,Ng[j]] = A^T * B_j [K,Ng[j]].
// bf16 only, every Ng[j] a multiple of 256 (gemm_tn_groups_supported says whether it applies).
bool gemm_tn_groups_supported(int dtype, int K, int ngroups, const int* Ng);
hipError_t launch_gemm_tn_groups(const void* A, int K, int M, int ngroups, const void* const* Bg,
                                 void* const* Cg, const int* Ng, hipStream_t st, float beta = 0.f,
                                 bool c_f32 = false, const int32_t* n_dev = nullptr);

// CUs of the current device (cached per device ordinal; 256 if the query fails)
inline int compute_units() {
    static std::atomic<int> cache[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    std::atomic<int>& c = cache[dev & 63];
    int n = c.load(std::memory_order_relaxed);
    if (n == 0) {
        int v = 0;
        n = (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) ? v : 256;
        c.store(n, std::memory_order_relaxed);
    }
    return n;
}

}  // namespace cf
