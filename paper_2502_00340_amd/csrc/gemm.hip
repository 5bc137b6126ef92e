// Dimension-reduced dense GEMMs (Sec. 3.2): next-node gradient dX = dY * W^T and
// parameter gradient dW = X^T * dY on kept rows only.
//
//   mode NT: C[M,N] = sum_seg A[M,K] * B[N,K]^T   (both operands contiguous along K)
//   mode TN: C[M,N] = sum_seg A[K,M]^T * B[K,N]   (both operands contiguous along M / N;
//                                                  K is the kept-token dimension)
// Up to three (A, B, K) segments accumulate into one output tile, which sums
// the gradients of a tensor consumed by several linears without rounding in
// between (e.g. d_gate*Wg^T + d_up*Wu^T).
//
// bf16 path: 32x32x16 bf16 MFMA, fp32 accumulators, 256 threads = 2x2 waves,
// block tile (2*TM*32) x (2*TN*32) x 64, double-buffered LDS, global loads of
// the next K-step issued before the MFMAs of the current one.
//   NT tiles sit in LDS as [row][64] with the 16-byte chunk index XOR-swizzled
//   by the row so that the 16 lanes of a ds_read_b128 hit distinct banks.
//   TN tiles sit in LDS exactly as in memory ([k][m]); a lane reads, for 8
//   consecutive k, the TM (TN) adjacent m (n) values it owns and transposes the
//   8 x TM block of 16-bit values in registers.  Fragment i of a lane then
//   belongs to output row  slot*TM + i  instead of  i*32 + slot; the epilogue
//   undoes this, and gets TN adjacent columns per lane to store together.
// fp32 path (check mode): plain LDS-tiled FMA kernel.
#include <type_traits>

#include "common.h"

namespace cf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

struct GemmArgs {
    const void* A[3];
    const void* B[3];
    int K[3];
    int nseg;
    void* C;
    int M, N;
    float beta;
};

static constexpr int BK = 64;

// ---- LDS addressing for NT tiles: row pitch 128 B, 8 chunks of 16 B ----------
__device__ __forceinline__ int nt_lds_off(int row, int chunk) {
    return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
}

template <int MODE, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
    constexpr int A_LD = BM / 32, B_LD = BN / 32;   // 16-byte chunks per thread per tile
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int slot = lane & 31, hh = lane >> 5;

    // tile mapping: consecutive blocks walk down M inside a band of 8 N-tiles... keep simple:
    const int tiles_m = (g.M + BM - 1) / BM;
    const int bm = blockIdx.x % tiles_m, bn = blockIdx.x / tiles_m;
    const int m0 = bm * BM, n0 = bn * BN;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 ra[A_LD], rb[B_LD];

    int total_steps = 0;
    for (int s = 0; s < g.nseg; ++s) total_steps += (g.K[s] + BK - 1) / BK;

    // ---- global -> registers for K-step (seg, k0) --------------------------
    auto load_global = [&](int seg, int k0) {
        const bf16_t* A = static_cast<const bf16_t*>(g.A[seg]);
        const bf16_t* B = static_cast<const bf16_t*>(g.B[seg]);
        const int K = g.K[seg];
        if (MODE == 0) {
            const int c = tid & 7, kk = k0 + c * 8;
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const int row = (tid >> 3) + 32 * i;
                const bool ok = (m0 + row < g.M) && (kk < K);
                ra[i] = ok ? *reinterpret_cast<const uint4*>(A + (int64_t)(m0 + row) * K + kk)
                           : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < B_LD; ++i) {
                const int row = (tid >> 3) + 32 * i;
                const bool ok = (n0 + row < g.N) && (kk < K);
                rb[i] = ok ? *reinterpret_cast<const uint4*>(B + (int64_t)(n0 + row) * K + kk)
                           : make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const int q = tid + 256 * i;
                const int kr = q / (BM / 8), c = q % (BM / 8);
                const bool ok = (k0 + kr < K) && (m0 + c * 8 < g.M);
                ra[i] = ok ? *reinterpret_cast<const uint4*>(A + (int64_t)(k0 + kr) * g.M + m0 + c * 8)
                           : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < B_LD; ++i) {
                const int q = tid + 256 * i;
                const int kr = q / (BN / 8), c = q % (BN / 8);
                const bool ok = (k0 + kr < K) && (n0 + c * 8 < g.N);
                rb[i] = ok ? *reinterpret_cast<const uint4*>(B + (int64_t)(k0 + kr) * g.N + n0 + c * 8)
                           : make_uint4(0, 0, 0, 0);
            }
        }
    };

    auto store_lds = [&](int stage) {
        unsigned char* sa = smem + stage * STAGE;
        unsigned char* sb = sa + A_BYTES;
        if (MODE == 0) {
            const int c = tid & 7;
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                *reinterpret_cast<uint4*>(sa + nt_lds_off((tid >> 3) + 32 * i, c)) = ra[i];
#pragma unroll
            for (int i = 0; i < B_LD; ++i)
                *reinterpret_cast<uint4*>(sb + nt_lds_off((tid >> 3) + 32 * i, c)) = rb[i];
        } else {
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                *reinterpret_cast<uint4*>(sa + (tid + 256 * i) * 16) = ra[i];
#pragma unroll
            for (int i = 0; i < B_LD; ++i)
                *reinterpret_cast<uint4*>(sb + (tid + 256 * i) * 16) = rb[i];
        }
    };

    // ---- fragments of one 16-wide K sub-step ---------------------------------
    auto load_frags_nt = [&](const unsigned char* tile, int row0, int ks, auto& frag, auto ntiles) {
        constexpr int NT_ = decltype(ntiles)::value;
#pragma unroll
        for (int i = 0; i < NT_; ++i) {
            const uint4 v = *reinterpret_cast<const uint4*>(tile + nt_lds_off(row0 + i * 32 + slot, ks * 2 + hh));
            frag[i] = __builtin_bit_cast(bf16x8_t, v);
        }
    };
    // tile is [64][W] bf16 as in memory; the lane owns columns col0 + slot*NT_ .. +NT_-1
    auto load_frags_tn = [&](const unsigned char* tile, int W, int col0, int ks, auto& frag, auto ntiles) {
        constexpr int NT_ = decltype(ntiles)::value;
        static_assert(NT_ == 2 || NT_ == 4, "TM/TN must be 2 or 4");
        unsigned r[8][NT_ / 2];
        const unsigned char* p = tile + ((ks * 16 + hh * 8) * W + col0 + slot * NT_) * 2;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (NT_ == 4) {
                const uint2 v = *reinterpret_cast<const uint2*>(p + e * W * 2);
                r[e][0] = v.x;
                r[e][NT_ / 2 - 1] = v.y;
            } else {
                r[e][0] = *reinterpret_cast<const unsigned*>(p + e * W * 2);
            }
        }
#pragma unroll
        for (int i = 0; i < NT_; ++i) {
            uint4 v;
            unsigned w[4];
#pragma unroll
            for (int pq = 0; pq < 4; ++pq) {
                const unsigned lo = r[2 * pq][i >> 1], hi = r[2 * pq + 1][i >> 1];
                w[pq] = (i & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
            }
            v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3];
            frag[i] = __builtin_bit_cast(bf16x8_t, v);
        }
    };

    auto compute = [&](int stage) {
        const unsigned char* sa = smem + stage * STAGE;
        const unsigned char* sb = sa + A_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t fa[TM], fb[TN];
            if (MODE == 0) {
                load_frags_nt(sa, wm * TM * 32, ks, fa, std::integral_constant<int, TM>());
                load_frags_nt(sb, wn * TN * 32, ks, fb, std::integral_constant<int, TN>());
            } else {
                load_frags_tn(sa, BM, wm * TM * 32, ks, fa, std::integral_constant<int, TM>());
                load_frags_tn(sb, BN, wn * TN * 32, ks, fb, std::integral_constant<int, TN>());
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    };

    // ---- main loop over (segment, k0) steps, flattened ------------------------
    int seg = 0, k0 = 0;
    auto advance = [&]() {
        k0 += BK;
        if (k0 >= g.K[seg]) { k0 = 0; ++seg; }
    };
    if (total_steps > 0) {
        load_global(seg, k0);
        advance();
        store_lds(0);
        __syncthreads();
        for (int step = 0; step < total_steps; ++step) {
            const int cur = step & 1;
            const bool more = step + 1 < total_steps;
            if (more) { load_global(seg, k0); advance(); }
            compute(cur);
            if (more) store_lds(cur ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue ---------------------------------------------------------------
    bf16_t* C = static_cast<bf16_t*>(g.C);
    const float beta = g.beta;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rslot = 8 * (v >> 2) + 4 * hh + (v & 3);
            if (MODE == 0) {
                const int m = m0 + wm * TM * 32 + i * 32 + rslot;
                if (m < g.M) {
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const int n = n0 + wn * TN * 32 + j * 32 + slot;
                        if (n < g.N) {
                            bf16_t* p = C + (int64_t)m * g.N + n;
                            float val = acc[i][j][v];
                            if (beta != 0.f) val += beta * bf16_to_f32(*p);
                            *p = f32_to_bf16(val);
                        }
                    }
                }
            } else {
                const int m = m0 + wm * TM * 32 + rslot * TM + i;
                const int n = n0 + wn * TN * 32 + slot * TN;     // TN consecutive columns
                if (m < g.M && n < g.N) {                          // N is a multiple of 8 >= TN
                    bf16_t* p = C + (int64_t)m * g.N + n;
                    float val[TN];
#pragma unroll
                    for (int j = 0; j < TN; ++j) val[j] = acc[i][j][v];
                    if (beta != 0.f) {
#pragma unroll
                        for (int j = 0; j < TN; ++j) val[j] += beta * bf16_to_f32(p[j]);
                    }
                    if (TN == 4) {
                        uint2 o;
                        o.x = pack_bf16x2(val[0], val[1]);
                        o.y = pack_bf16x2(val[TN - 2], val[TN - 1]);
                        *reinterpret_cast<uint2*>(p) = o;
                    } else {
                        *reinterpret_cast<unsigned*>(p) = pack_bf16x2(val[0], val[1]);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// fp32 check-mode GEMM: 64x64 tile, 16-wide K step, 4x4 outputs per thread
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64 + 4];
    const int tid = threadIdx.x;
    const int tiles_m = (g.M + 63) / 64;
    const int m0 = (blockIdx.x % tiles_m) * 64, n0 = (blockIdx.x / tiles_m) * 64;
    const int tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    for (int s = 0; s < g.nseg; ++s) {
        const float* A = static_cast<const float*>(g.A[s]);
        const float* B = static_cast<const float*>(g.B[s]);
        const int K = g.K[s];
        for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tid + 256 * i;      // 0..1023
                int kk, r;
                if (MODE == 0) { kk = e & 15; r = e >> 4; } else { r = e & 63; kk = e >> 6; }
                const bool ka = k0 + kk < K;
                float av = 0.f, bv = 0.f;
                if (ka && m0 + r < g.M)
                    av = MODE == 0 ? A[(int64_t)(m0 + r) * K + k0 + kk] : A[(int64_t)(k0 + kk) * g.M + m0 + r];
                if (ka && n0 + r < g.N)
                    bv = MODE == 0 ? B[(int64_t)(n0 + r) * K + k0 + kk] : B[(int64_t)(k0 + kk) * g.N + n0 + r];
                As[kk][r] = av;
                Bs[kk][r] = bv;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
            }
            __syncthreads();
        }
    }
    float* C = static_cast<float*>(g.C);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= g.N) continue;
            float* p = C + (int64_t)m * g.N + n;
            *p = (g.beta != 0.f) ? acc[i][j] + g.beta * *p : acc[i][j];
        }
    }
}

template <int MODE, int TM, int TN>
static hipError_t launch_bf16(const GemmArgs& g, hipStream_t st) {
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    constexpr int smem = 2 * (BM + BN) * BK * 2;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<MODE, TM, TN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int grid = ceil_div(g.M, BM) * ceil_div(g.N, BN);
    gemm_bf16_kernel<MODE, TM, TN><<<grid, 256, smem, st>>>(g);
    return hipGetLastError();
}

hipError_t launch_gemm(int dtype, int mode, const GemmSeg* segs, int nseg, void* C, int M, int N,
                       float beta, hipStream_t st) {
    if (M <= 0 || N <= 0) return hipSuccess;
    GemmArgs g;
    g.nseg = 0;
    for (int s = 0; s < nseg; ++s) {
        if (segs[s].K <= 0) continue;
        g.A[g.nseg] = segs[s].A;
        g.B[g.nseg] = segs[s].B;
        g.K[g.nseg] = segs[s].K;
        ++g.nseg;
    }
    for (int s = g.nseg; s < 3; ++s) { g.A[s] = nullptr; g.B[s] = nullptr; g.K[s] = 0; }
    g.C = C; g.M = M; g.N = N; g.beta = beta;
    if (g.nseg == 0) {
        // empty contraction: C = beta*C; only beta in {0,1} is supported by the API
        if (beta == 0.f) return launch_fill_zero(C, (size_t)M * N * dtype_size(dtype), st);
        return hipSuccess;
    }
    if (dtype == CF_F32) {
        const int grid = ceil_div(M, 64) * ceil_div(N, 64);
        if (mode == 0) gemm_f32_kernel<0><<<grid, 256, 0, st>>>(g);
        else gemm_f32_kernel<1><<<grid, 256, 0, st>>>(g);
        return hipGetLastError();
    }
    // tile choice: big tiles when they still give every CU work, else 128x128
    const int64_t big_tiles = (int64_t)ceil_div(M, 256) * ceil_div(N, 256);
    const bool big = big_tiles >= 200;
    if (mode == 0) return big ? launch_bf16<0, 4, 4>(g, st) : launch_bf16<0, 2, 2>(g, st);
    return big ? launch_bf16<1, 4, 4>(g, st) : launch_bf16<1, 2, 2>(g, st);
}

}  // namespace cf
