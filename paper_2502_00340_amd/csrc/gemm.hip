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

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// Workgroup barrier that orders LDS traffic only: global loads that are still
// in flight (the register prefetch of a later K-step) stay in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

#define CF_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Buffer resource over [base, base+bytes): loads past the end return zeros, which is
// how ragged tiles are predicated without branches.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, int64_t bytes) {
    const int64_t lim = bytes < 0 ? 0 : (bytes > 0xFFFFFFFFll ? 0xFFFFFFFFll : bytes);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)(unsigned)lim, 0x00020000);
}

// Tile order: consecutive logical tiles form bands of GROUP_M tile rows walked
// column by column, and each of the 8 XCDs (block id mod 8) takes one contiguous
// run of logical tiles, so the blocks resident on one XCD share operand panels
// in that XCD's L2.
__device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int& bm, int& bn) {
    constexpr int GROUP_M = 8;
    const int nb = tiles_m * tiles_n;
    const int xcd = pid & 7, local = pid >> 3;
    const int base = nb >> 3, rem = nb & 7;
    const int l = xcd * base + (xcd < rem ? xcd : rem) + local;
    const int band = l / (GROUP_M * tiles_n);
    const int first_m = band * GROUP_M;
    const int gsize = min(GROUP_M, tiles_m - first_m);
    const int r = l - band * GROUP_M * tiles_n;
    bm = first_m + r % gsize;
    bn = r / gsize;
}

template <int MODE, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
    constexpr int A_LD = BM / 32, B_LD = BN / 32;   // 16-byte chunks per thread per tile
    constexpr unsigned OOB = 0xFFFFFFFFu;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int slot = lane & 31, hh = lane >> 5;

    int bm, bn;
    tile_coords(blockIdx.x, (g.M + BM - 1) / BM, (g.N + BN - 1) / BN, bm, bn);
    const int m0 = bm * BM, n0 = bn * BN;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    int total_steps = 0;
    for (int s = 0; s < g.nseg; ++s) total_steps += (g.K[s] + BK - 1) / BK;

    // ---- global -> registers: one K-step of both operand tiles -----------------
    // Offsets are relative to the block's first row/column so they fit 32 bits.
    u32x4_t ra[A_LD], rb[B_LD];
    int seg = 0, k0 = 0;                 // K-step the NEXT issue_global() fetches
    __amdgpu_buffer_rsrc_t rsA, rsB;
    auto open_segment = [&](int s) {
        const bf16_t* A = static_cast<const bf16_t*>(g.A[s]);
        const bf16_t* B = static_cast<const bf16_t*>(g.B[s]);
        const int64_t K = g.K[s];
        if (MODE == 0) {
            rsA = make_rsrc(A + (int64_t)m0 * K, ((int64_t)g.M - m0) * K * 2);
            rsB = make_rsrc(B + (int64_t)n0 * K, ((int64_t)g.N - n0) * K * 2);
        } else {
            rsA = make_rsrc(A + m0, (K * g.M - m0) * 2);
            rsB = make_rsrc(B + n0, (K * g.N - n0) * 2);
        }
    };
    auto issue_global = [&]() {
        const int K = g.K[seg];
        if (MODE == 0) {
            const int c = tid & 7;
            const unsigned kb = (k0 + c * 8 < K) ? (unsigned)(k0 + c * 8) * 2u : OOB;
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const unsigned row = (tid >> 3) + 32 * i;
                ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsA, kb == OOB ? OOB : row * (unsigned)K * 2u + kb, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < B_LD; ++i) {
                const unsigned row = (tid >> 3) + 32 * i;
                rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rsB, kb == OOB ? OOB : row * (unsigned)K * 2u + kb, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const int q = tid + 256 * i;
                const int kr = q / (BM / 8), c = q % (BM / 8);
                const unsigned off = (unsigned)(k0 + kr) * (unsigned)g.M * 2u + c * 16u;
                ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rsA, (m0 + c * 8 < g.M && k0 + kr < K) ? off : OOB, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < B_LD; ++i) {
                const int q = tid + 256 * i;
                const int kr = q / (BN / 8), c = q % (BN / 8);
                const unsigned off = (unsigned)(k0 + kr) * (unsigned)g.N * 2u + c * 16u;
                rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rsB, (n0 + c * 8 < g.N && k0 + kr < K) ? off : OOB, 0, 0);
            }
        }
        k0 += BK;
        if (k0 >= K) {
            k0 = 0;
            ++seg;
            if (seg < g.nseg) open_segment(seg);
        }
    };

    auto store_lds = [&](int stage) {
        unsigned char* sa = smem + stage * STAGE;
        unsigned char* sb = sa + A_BYTES;
        if (MODE == 0) {
            const int c = tid & 7;
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                *reinterpret_cast<u32x4_t*>(sa + nt_lds_off((tid >> 3) + 32 * i, c)) = ra[i];
#pragma unroll
            for (int i = 0; i < B_LD; ++i)
                *reinterpret_cast<u32x4_t*>(sb + nt_lds_off((tid >> 3) + 32 * i, c)) = rb[i];
        } else {
#pragma unroll
            for (int i = 0; i < A_LD; ++i)
                *reinterpret_cast<u32x4_t*>(sa + (tid + 256 * i) * 16) = ra[i];
#pragma unroll
            for (int i = 0; i < B_LD; ++i)
                *reinterpret_cast<u32x4_t*>(sb + (tid + 256 * i) * 16) = rb[i];
        }
    };

    // ---- LDS -> MFMA fragments of one 16-wide K sub-step ------------------------
    struct Frags {
        bf16x8_t a[TM], b[TN];
    };
    auto frags_nt = [&](const unsigned char* tile, int row0, int ks, bf16x8_t* frag, auto ntiles) {
        constexpr int NT_ = decltype(ntiles)::value;
#pragma unroll
        for (int i = 0; i < NT_; ++i)
            frag[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(
                                                       tile + nt_lds_off(row0 + i * 32 + slot, ks * 2 + hh)));
    };
    // tile is [64][W] bf16 as in memory; the lane owns columns col0 + slot*NT_ .. +NT_-1
    auto frags_tn = [&](const unsigned char* tile, int W, int col0, int ks, bf16x8_t* frag, auto ntiles) {
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
            u32x4_t v;
#pragma unroll
            for (int pq = 0; pq < 4; ++pq) {
                const unsigned lo = r[2 * pq][i >> 1], hi = r[2 * pq + 1][i >> 1];
                v[pq] = (i & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
            }
            frag[i] = __builtin_bit_cast(bf16x8_t, v);
        }
    };
    auto load_frags = [&](int stage, int ks, Frags& f) {
        const unsigned char* sa = smem + stage * STAGE;
        const unsigned char* sb = sa + A_BYTES;
        if (MODE == 0) {
            frags_nt(sa, wm * TM * 32, ks, f.a, std::integral_constant<int, TM>());
            frags_nt(sb, wn * TN * 32, ks, f.b, std::integral_constant<int, TN>());
        } else {
            frags_tn(sa, BM, wm * TM * 32, ks, f.a, std::integral_constant<int, TM>());
            frags_tn(sb, BN, wn * TN * 32, ks, f.b, std::integral_constant<int, TN>());
        }
    };
    auto mma = [&](const Frags& f) {
#ifdef CF_EXP_NOMMA
        if (g.beta == 123.f)
#endif
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
    };

    // ---- software-pipelined main loop ----------------------------------------------
    // Iteration t multiplies tile t out of LDS stage t&1 while
    //   * tile t+1 (fetched into registers during iteration t-1) is written to the other stage,
    //   * tile t+2 is fetched from global memory into the same registers,
    //   * fragments of the next 16-wide sub-step are read from LDS ahead of the MFMAs that
    //     use the current ones.
    // One LDS barrier per iteration, placed before the last sub-step so that the first
    // fragments of tile t+1 are already on their way when iteration t+1 starts.
    if (total_steps > 0) {
        Frags f0, f1;
        open_segment(0);
        issue_global();
        store_lds(0);
        if (total_steps > 1) issue_global();
        lds_barrier();
        load_frags(0, 0, f0);
        for (int t = 0; t < total_steps; ++t) {
            const int cur = t & 1;
#ifndef CF_EXP_NOSTORE
            if (t + 1 < total_steps) store_lds(cur ^ 1);
#endif
#ifndef CF_EXP_NOGLOBAL
            if (t + 2 < total_steps) issue_global();
#endif
            CF_SCHED_FENCE();
            load_frags(cur, 1, f1);
            CF_SCHED_FENCE();
            mma(f0);
            CF_SCHED_FENCE();
            load_frags(cur, 2, f0);
            CF_SCHED_FENCE();
            mma(f1);
            CF_SCHED_FENCE();
            load_frags(cur, 3, f1);
            CF_SCHED_FENCE();
            mma(f0);
            CF_SCHED_FENCE();
            lds_barrier();
            if (t + 1 < total_steps) load_frags(cur ^ 1, 0, f0);
            CF_SCHED_FENCE();
            mma(f1);
            CF_SCHED_FENCE();
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
