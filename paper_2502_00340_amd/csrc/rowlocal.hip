// Row-local backward operators on kept rows (Sec. 3.2: element-wise products
// of a row-sparse gradient inherit its row sparsity).  Every kernel takes an
// optional kept-row index for tensors that are still stored full length, so
// the gather of those tensors is folded into the read.  Arithmetic is fp32;
// storage is fp32 or bf16.  All of them are HBM-bound streaming kernels.
#include "common.h"

namespace cf {

__device__ __forceinline__ float sigmoidf_(float z) { return 1.0f / (1.0f + __expf(-z)); }

// d_gate = d_act * up * s(1 + gate(1-s)), d_up = d_act * gate * s,  s = sigmoid(gate);
// act (nullable) = gate * s * up, the SwiGLU product rebuilt in the same pass.
// d_gate may alias d_act (every element is read before it is written, by the same thread).
// copy_src (nullable): after its share of the SwiGLU elements every thread also copies its share of
// copy_dst[j, :] = copy_src[idx[j], :] (copy_cols columns, a multiple of VN): the kept rows of the
// upstream gradient, which the down projection's parameter-gradient GEMM contracts over; folding the
// copy in here saves the launch of a gather kernel.
template <typename T>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const T* d_act,
                                                         const T* __restrict__ gate,
                                                         const T* __restrict__ up,
                                                         const int32_t* __restrict__ idx,
                                                         int n_max, const int32_t* __restrict__ n_dev, int F, T* d_gate,
                                                         T* __restrict__ d_up, T* __restrict__ act,
                                                         const T* __restrict__ copy_src, int copy_cols,
                                                         T* __restrict__ copy_dst) {
    constexpr int VN = Vec<T>::N;
    const int n_rows = live_rows(n_max, n_dev);
    if (copy_src != nullptr) {
        const int cvpr = copy_cols / VN;
        const int64_t ctotal = (int64_t)n_rows * cvpr;
        for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < ctotal; v += (int64_t)gridDim.x * 256) {
            const int j = (int)(v / cvpr);
            const int c = (int)(v % cvpr) * VN;
            *reinterpret_cast<uint4*>(copy_dst + (int64_t)j * copy_cols + c) =
                *reinterpret_cast<const uint4*>(copy_src + (int64_t)idx[j] * copy_cols + c);
        }
    }
    const int vpr = F / VN;
    const int64_t total = (int64_t)n_rows * vpr;
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < total; v += (int64_t)gridDim.x * 256) {
        const int j = (int)(v / vpr);
        const int c = (int)(v % vpr) * VN;
        const int64_t row = idx ? idx[j] : j;
        float g[VN], u[VN], da[VN], dg[VN], du[VN], a[VN];
        Vec<T>::load(gate + row * F + c, g);
        Vec<T>::load(up + row * F + c, u);
        Vec<T>::load(d_act + (int64_t)j * F + c, da);
#pragma unroll
        for (int e = 0; e < VN; ++e) {
            const float s = sigmoidf_(g[e]);
            dg[e] = da[e] * u[e] * s * (1.0f + g[e] * (1.0f - s));
            du[e] = da[e] * g[e] * s;
            a[e] = g[e] * s * u[e];
        }
        Vec<T>::store(d_gate + (int64_t)j * F + c, dg);
        Vec<T>::store(d_up + (int64_t)j * F + c, du);
        if (act) Vec<T>::store(act + (int64_t)j * F + c, a);
    }
}

static constexpr int RMS_MAX_VEC = 8;   // 16-byte vectors per thread: H <= 256*8*VN

__device__ __forceinline__ void block_sum2(float& a, float& b, float* red /*8 floats*/) {
    a = wave_sum(a);
    b = wave_sum(b);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { red[wave] = a; red[4 + wave] = b; }
    __syncthreads();
    a = red[0] + red[1] + red[2] + red[3];
    b = red[4] + red[5] + red[6] + red[7];
}

// h[j,:] = x[row,:] * rstd * g,  rstd = (mean(x^2) + eps)^-1/2
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const T* __restrict__ x,
                                                          const T* __restrict__ g,
                                                          const int32_t* __restrict__ idx,
                                                          int n_max, const int32_t* __restrict__ n_dev, int H, float eps,
                                                          T* __restrict__ h) {
    constexpr int VN = Vec<T>::N;
    __shared__ float red[8];
    const int n_rows = live_rows(n_max, n_dev);
    const int vpr = H / VN;
    for (int j = blockIdx.x; j < n_rows; j += gridDim.x) {
        const int64_t row = idx ? idx[j] : j;
        float xv[RMS_MAX_VEC][VN];
        float ss = 0.f, dummy = 0.f;
#pragma unroll
        for (int i = 0; i < RMS_MAX_VEC; ++i) {
            const int v = threadIdx.x + i * 256;
            if (v < vpr) {
                Vec<T>::load(x + row * H + v * VN, xv[i]);
#pragma unroll
                for (int e = 0; e < VN; ++e) ss += xv[i][e] * xv[i][e];
            }
        }
        block_sum2(ss, dummy, red);
        const float rstd = rsqrtf(ss / (float)H + eps);
#pragma unroll
        for (int i = 0; i < RMS_MAX_VEC; ++i) {
            const int v = threadIdx.x + i * 256;
            if (v < vpr) {
                float gv[VN], o[VN];
                Vec<T>::load(g + v * VN, gv);
#pragma unroll
                for (int e = 0; e < VN; ++e) o[e] = xv[i][e] * rstd * gv[e];
                Vec<T>::store(h + (int64_t)j * H + v * VN, o);
            }
        }
    }
}

// dx_out[j,:] = res[j,:] + rstd*(u - n*mean(u*n)),  n = x*rstd, u = dh*g
// dg_partial[block,:] = sum over the block's rows of dh*n
// h_out (nullable): h_out[j,:] = n*g, the normalised row itself (what rmsnorm_fwd_kernel computes, with
// the same arithmetic): the parameter-gradient GEMMs of the linears behind this norm need it as an
// operand, and the row and its rstd are in registers here anyway.
// A block owns one row at a time, NV 16-byte vectors per thread, and works on two rows per
// iteration so that the loads of the second row overlap the reduction of the first; every
// load of an iteration (x, dh, res of both rows) is issued before the first reduction.
// The rows are dealt out to rmsnorm_bwd_nblk(live rows) blocks whatever the grid is (a grid sized for
// an upper bound of the row count leaves the blocks past that number idle), so the partial sums, and
// with them the rounding of the gain gradient, depend on the number of live rows alone.
__host__ __device__ inline int rmsnorm_bwd_nblk(int n_rows) {
    const int pairs = (n_rows + 1) / 2;             // a block takes two rows per iteration
    return pairs < 512 ? pairs : 512;
}

template <typename T, int NV>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const T* __restrict__ dh,
                                                          const T* __restrict__ x,
                                                          const T* __restrict__ g,
                                                          const int32_t* __restrict__ idx,
                                                          const T* __restrict__ res, int n_max,
                                                          const int32_t* __restrict__ n_dev,
                                                          int H, float eps, T* __restrict__ dx_out,
                                                          float* __restrict__ dg_partial, T* __restrict__ h_out) {
    constexpr int VN = Vec<T>::N;
    __shared__ float red[16];
    const int n_rows = live_rows(n_max, n_dev);
    const int nblk = rmsnorm_bwd_nblk(n_rows);
    if ((int)blockIdx.x >= nblk) return;
    const int vpr = H / VN;
    float gv[NV][VN], dgacc[NV][VN];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = threadIdx.x + i * 256;
#pragma unroll
        for (int e = 0; e < VN; ++e) { dgacc[i][e] = 0.f; gv[i][e] = 0.f; }
        if (v < vpr) Vec<T>::load(g + v * VN, gv[i]);
    }
    const int wave = threadIdx.x >> 6;
    for (int j0 = blockIdx.x * 2; j0 < n_rows; j0 += nblk * 2) {
        float xv[2][NV][VN], dv[2][NV][VN], rv[2][NV][VN];
        float ss[2] = {0.f, 0.f}, sd[2] = {0.f, 0.f};
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int j = j0 + r;
            const bool live = j < n_rows;
            const int64_t row = live ? (idx ? idx[j] : j) : 0;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int v = threadIdx.x + i * 256;
                if (live && v < vpr) {
                    Vec<T>::load(x + row * H + v * VN, xv[r][i]);
                    Vec<T>::load(dh + (int64_t)j * H + v * VN, dv[r][i]);
                    Vec<T>::load(res + (int64_t)j * H + v * VN, rv[r][i]);
                } else {
#pragma unroll
                    for (int e = 0; e < VN; ++e) { xv[r][i][e] = 0.f; dv[r][i][e] = 0.f; rv[r][i][e] = 0.f; }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < NV; ++i)
#pragma unroll
                for (int e = 0; e < VN; ++e) {
                    ss[r] += xv[r][i][e] * xv[r][i][e];
                    sd[r] += dv[r][i][e] * gv[i][e] * xv[r][i][e];
                }
#pragma unroll
        for (int r = 0; r < 2; ++r) { ss[r] = wave_sum(ss[r]); sd[r] = wave_sum(sd[r]); }
        __syncthreads();
        if ((threadIdx.x & 63) == 0) {
            red[wave] = ss[0]; red[4 + wave] = sd[0]; red[8 + wave] = ss[1]; red[12 + wave] = sd[1];
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int j = j0 + r;
            if (j >= n_rows) break;
            const float ssr = red[8 * r] + red[8 * r + 1] + red[8 * r + 2] + red[8 * r + 3];
            const float sdr = red[8 * r + 4] + red[8 * r + 5] + red[8 * r + 6] + red[8 * r + 7];
            const float rstd = rsqrtf(ssr / (float)H + eps);
            const float c = sdr * rstd / (float)H;          // mean(u*n)
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int v = threadIdx.x + i * 256;
                if (v < vpr) {
                    float o[VN];
#pragma unroll
                    for (int e = 0; e < VN; ++e) {
                        const float n = xv[r][i][e] * rstd;
                        o[e] = rv[r][i][e] + rstd * (dv[r][i][e] * gv[i][e] - n * c);
                        dgacc[i][e] += dv[r][i][e] * n;
                    }
                    Vec<T>::store(dx_out + (int64_t)j * H + v * VN, o);
                    if (h_out != nullptr) {
#pragma unroll
                        for (int e = 0; e < VN; ++e) o[e] = xv[r][i][e] * rstd * gv[i][e];
                        Vec<T>::store(h_out + (int64_t)j * H + v * VN, o);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int v = threadIdx.x + i * 256;
        if (v < vpr) {
#pragma unroll
            for (int e = 0; e < VN; ++e) dg_partial[(int64_t)blockIdx.x * H + v * VN + e] = dgacc[i][e];
        }
    }
}

// out[c] = sum_b partial[b,c]: a block owns 32 columns (8 lanes x 4 columns), 32 row groups
// stride through the partials with 16-byte loads, many in flight; H is a multiple of 4.
// The order of the additions is fixed, so the result is reproducible.  ACC: out is fp32 and the
// sum is added to it (main-gradient accumulation).
template <typename T, bool ACC = false>
__global__ __launch_bounds__(256) void colsum_finish_kernel(const float* __restrict__ partial,
                                                            int n_max, const int32_t* __restrict__ n_dev, int H,
                                                            T* __restrict__ out) {
    __shared__ float red[32][33];
    const int nblk = rmsnorm_bwd_nblk(live_rows(n_max, n_dev));     // the partials that the backward kernel wrote
    const int cq = threadIdx.x & 7, rg = threadIdx.x >> 3;
    const int c = blockIdx.x * 32 + cq * 4;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    if (c < H) {
#pragma unroll 8
        for (int b = rg; b < nblk; b += 32) {
            const float4 v = *reinterpret_cast<const float4*>(partial + (int64_t)b * H + c);
            s[0] += v.x; s[1] += v.y; s[2] += v.z; s[3] += v.w;
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) red[rg][cq * 4 + e] = s[e];
    __syncthreads();
    if (threadIdx.x < 32 && blockIdx.x * 32 + threadIdx.x < H) {
        float t = 0.f;
#pragma unroll
        for (int r = 0; r < 32; ++r) t += red[r][threadIdx.x];
        if (ACC) out[blockIdx.x * 32 + threadIdx.x] += from_f32<T>(t);
        else out[blockIdx.x * 32 + threadIdx.x] = from_f32<T>(t);
    }
}

// D[j,h] = sum_c da[j,h*d+c] * a[row,h*d+c]   (the FlashAttention-backward row term), row = a_idx ?
// a_idx[j] : j.  With a_idx the pass also writes the compact copies a_out[j,:] = a[row,:] and, when
// q_src is given, q_out[j,:] = q_src[row,:] (the gathers of attn_out and q folded into this read).
template <typename T>
__global__ __launch_bounds__(256) void attn_rowdot_kernel(const T* __restrict__ da,
                                                          const T* __restrict__ a, int n_max,
                                                          const int32_t* __restrict__ n_dev,
                                                          int Hq, int d, float* __restrict__ D,
                                                          const int32_t* __restrict__ a_idx, T* __restrict__ a_out,
                                                          const T* __restrict__ q_src, T* __restrict__ q_out) {
    constexpr int VN = Vec<T>::N;
    const int n_rows = live_rows(n_max, n_dev);
    const int lanes = d / VN;                    // lanes per (row, head): power of two <= 64
    const int64_t total = (int64_t)n_rows * Hq * lanes;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    float s = 0.f;
    int64_t pair = gid / lanes;
    if (gid < total) {
        const int part = (int)(gid % lanes);
        int64_t src = pair;
        if (a_idx != nullptr) src = (int64_t)a_idx[pair / Hq] * Hq + pair % Hq;
        float p[VN], q[VN];
        Vec<T>::load(da + pair * d + part * VN, p);
        Vec<T>::load(a + src * d + part * VN, q);
#pragma unroll
        for (int e = 0; e < VN; ++e) s += p[e] * q[e];
        if (a_idx != nullptr) {
            Vec<T>::store(a_out + pair * d + part * VN, q);        // widening and rounding back is exact
            if (q_src != nullptr)
                *reinterpret_cast<uint4*>(q_out + pair * d + part * VN) =
                    *reinterpret_cast<const uint4*>(q_src + src * d + part * VN);
        }
    }
    for (int o = lanes >> 1; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (gid < total && (gid % lanes) == 0) D[pair] = s;
}

// Transposed rotary rotation, in place: for i < d/2 and c = cos[pos,i], s = sin[pos,i]
//   dx[i] = dy[i]*c + dy[i+d/2]*s,   dx[i+d/2] = dy[i+d/2]*c - dy[i]*s
// One thread per vector of VN frequencies of one (row, head); d/2 is a multiple of VN.
template <typename T>
__global__ __launch_bounds__(256) void rope_bwd_kernel(T* __restrict__ g, const int32_t* __restrict__ idx,
                                                       int n_max, const int32_t* __restrict__ n_dev, int heads, int d, int S,
                                                       const float* __restrict__ cs,
                                                       const float* __restrict__ sn) {
    constexpr int VN = Vec<T>::N;
    const int n_rows = live_rows(n_max, n_dev);
    const int half = d / 2, vph = half / VN;            // vectors per head half
    const int64_t total = (int64_t)n_rows * heads * vph;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        const int iv = (int)(t % vph);
        const int64_t rh = t / vph;
        const int h = (int)(rh % heads);
        const int64_t j = rh / heads;
        const int pos = (int)((idx ? (int64_t)idx[j] : j) % S);
        T* p = g + (j * heads + h) * d + iv * VN;
        float lo[VN], hi[VN], olo[VN], ohi[VN];
        Vec<T>::load(p, lo);
        Vec<T>::load(p + half, hi);
#pragma unroll
        for (int e = 0; e < VN; ++e) {
            const float c = cs[(int64_t)pos * half + iv * VN + e], s = sn[(int64_t)pos * half + iv * VN + e];
            olo[e] = lo[e] * c + hi[e] * s;
            ohi[e] = hi[e] * c - lo[e] * s;
        }
        Vec<T>::store(p, olo);
        Vec<T>::store(p + half, ohi);
    }
}

// ---------------------------------------------------------------------------

static int stream_grid(int64_t vec_total) {
    int64_t g = (vec_total + 255) / 256;
    if (g > 256 * 32) g = 256 * 32;
    if (g < 1) g = 1;
    return (int)g;
}

hipError_t launch_swiglu_bwd(int dtype, const void* d_act, const void* gate, const void* up,
                             const int32_t* idx, RowCount rows, int F, void* d_gate, void* d_up,
                             void* act, hipStream_t st, const void* copy_src, int copy_cols, void* copy_dst) {
    const int n_rows = rows.n;
    if (n_rows <= 0) return hipSuccess;
    if (copy_src != nullptr && idx == nullptr) return hipErrorInvalidValue;
    if (dtype == CF_F32)
        swiglu_bwd_kernel<float><<<stream_grid((int64_t)n_rows * F / 4), 256, 0, st>>>(
            (const float*)d_act, (const float*)gate, (const float*)up, idx, n_rows, rows.dev, F,
            (float*)d_gate, (float*)d_up, (float*)act, (const float*)copy_src, copy_cols, (float*)copy_dst);
    else
        swiglu_bwd_kernel<bf16_t><<<stream_grid((int64_t)n_rows * F / 8), 256, 0, st>>>(
            (const bf16_t*)d_act, (const bf16_t*)gate, (const bf16_t*)up, idx, n_rows, rows.dev, F,
            (bf16_t*)d_gate, (bf16_t*)d_up, (bf16_t*)act, (const bf16_t*)copy_src, copy_cols, (bf16_t*)copy_dst);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_fwd(int dtype, const void* x, const void* g, const int32_t* idx,
                              RowCount rows, int H, float eps, void* h, hipStream_t st) {
    const int n_rows = rows.n;
    if (n_rows <= 0) return hipSuccess;
    const int grid = n_rows < 256 * 16 ? n_rows : 256 * 16;
    if (dtype == CF_F32)
        rmsnorm_fwd_kernel<float><<<grid, 256, 0, st>>>((const float*)x, (const float*)g, idx,
                                                        n_rows, rows.dev, H, eps, (float*)h);
    else
        rmsnorm_fwd_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)x, (const bf16_t*)g, idx,
                                                         n_rows, rows.dev, H, eps, (bf16_t*)h);
    return hipGetLastError();
}

int rmsnorm_bwd_blocks(int n_rows) {
    return n_rows < 1 ? 1 : rmsnorm_bwd_nblk(n_rows);
}

template <typename T>
static void rmsnorm_bwd_dispatch(int nv, int nblk, hipStream_t st, const void* dh, const void* x, const void* g,
                                 const int32_t* idx, const void* res, RowCount rows, int H, float eps,
                                 void* dx_out, float* dg_partial, void* h_out) {
#define CF_RMS_BWD(NV)                                                                               \
    rmsnorm_bwd_kernel<T, NV><<<nblk, 256, 0, st>>>((const T*)dh, (const T*)x, (const T*)g, idx,      \
                                                    (const T*)res, rows.n, rows.dev, H, eps, (T*)dx_out, dg_partial, (T*)h_out)
    if (nv <= 1) CF_RMS_BWD(1);
    else if (nv <= 2) CF_RMS_BWD(2);
    else if (nv <= 4) CF_RMS_BWD(4);
    else CF_RMS_BWD(8);
#undef CF_RMS_BWD
}

hipError_t launch_rmsnorm_bwd(int dtype, const void* dh, const void* x, const void* g,
                              const int32_t* idx, const void* res, RowCount rows, int H, float eps,
                              void* dx_out, float* dg_partial, void* dg_out, hipStream_t st, bool dg_acc_f32,
                              void* h_out) {
    const int n_rows = rows.n;
    const int nblk = rmsnorm_bwd_blocks(n_rows);
    if (n_rows <= 0) return dg_acc_f32 ? hipSuccess : launch_fill_zero(dg_out, (size_t)H * dtype_size(dtype), st);
    const int vn = dtype == CF_F32 ? 4 : 8;
    const int nv = ceil_div(H / vn, 256);           // 16-byte vectors per thread (<= RMS_MAX_VEC, checked by the API)
    const int fin = ceil_div(H, 32);
    if (dtype == CF_F32) {
        rmsnorm_bwd_dispatch<float>(nv, nblk, st, dh, x, g, idx, res, rows, H, eps, dx_out, dg_partial, h_out);
        if (dg_acc_f32) colsum_finish_kernel<float, true><<<fin, 256, 0, st>>>(dg_partial, n_rows, rows.dev, H, (float*)dg_out);
        else colsum_finish_kernel<float><<<fin, 256, 0, st>>>(dg_partial, n_rows, rows.dev, H, (float*)dg_out);
    } else {
        rmsnorm_bwd_dispatch<bf16_t>(nv, nblk, st, dh, x, g, idx, res, rows, H, eps, dx_out, dg_partial, h_out);
        if (dg_acc_f32) colsum_finish_kernel<float, true><<<fin, 256, 0, st>>>(dg_partial, n_rows, rows.dev, H, (float*)dg_out);
        else colsum_finish_kernel<bf16_t><<<fin, 256, 0, st>>>(dg_partial, n_rows, rows.dev, H, (bf16_t*)dg_out);
    }
    return hipGetLastError();
}

hipError_t launch_rope_bwd(int dtype, void* g, const int32_t* idx, RowCount rows, int heads, int d, int S,
                           const float* cos, const float* sin, hipStream_t st) {
    const int n_rows = rows.n;
    if (n_rows <= 0) return hipSuccess;
    const int vn = dtype == CF_F32 ? 4 : 8;
    if ((d / 2) % vn != 0) return hipErrorInvalidValue;
    const int64_t total = (int64_t)n_rows * heads * (d / 2 / vn);
    if (dtype == CF_F32)
        rope_bwd_kernel<float><<<stream_grid(total), 256, 0, st>>>((float*)g, idx, n_rows, rows.dev, heads, d, S, cos, sin);
    else
        rope_bwd_kernel<bf16_t><<<stream_grid(total), 256, 0, st>>>((bf16_t*)g, idx, n_rows, rows.dev, heads, d, S, cos, sin);
    return hipGetLastError();
}

hipError_t launch_attn_rowdot(int dtype, const void* da, const void* a, RowCount rows, int Hq, int d,
                              float* D, hipStream_t st, const int32_t* a_idx, void* a_out, const void* q_src,
                              void* q_out) {
    const int n_rows = rows.n;
    if (n_rows <= 0) return hipSuccess;
    const int vn = dtype == CF_F32 ? 4 : 8;
    const int64_t total = (int64_t)n_rows * Hq * (d / vn);
    const int grid = (int)((total + 255) / 256);
    if (dtype == CF_F32)
        attn_rowdot_kernel<float><<<grid, 256, 0, st>>>((const float*)da, (const float*)a, n_rows, rows.dev, Hq, d, D,
                                                        a_idx, (float*)a_out, (const float*)q_src, (float*)q_out);
    else
        attn_rowdot_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)da, (const bf16_t*)a, n_rows, rows.dev, Hq, d, D,
                                                         a_idx, (bf16_t*)a_out, (const bf16_t*)q_src, (bf16_t*)q_out);
    return hipGetLastError();
}

}  // namespace cf
