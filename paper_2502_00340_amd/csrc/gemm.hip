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
// block tile (2*TM*32) x (2*TN*32), K step 32, four LDS stages.
//   * Operand tiles go from global memory straight into LDS (buffer_load ... lds,
//     16 bytes per lane, no register hop); three K-steps are in flight while one
//     is multiplied.  Ragged edges come from the buffer descriptor's range check,
//     which returns zeros, so there are no branches around loads.
//   * One LDS barrier per K-step, placed between the two 16-wide sub-steps, and the
//     fragments of the next sub-step are read ahead of the MFMAs of the current one.
//   * NT tiles sit in LDS as [row][32] (64-byte rows) with the 16-byte chunk index
//     XOR-ed with (row/4)%4, which makes the 16 lanes of a ds_read_b128 hit distinct
//     banks; a lane of the loading wave picks the global chunk that belongs in its
//     (fixed) LDS slot.
//   * TN tiles sit in LDS exactly as in memory ([k][m]); a lane reads, for 8
//     consecutive k, the TM (TN) adjacent m (n) values it owns and transposes the
//     8 x TM block of 16-bit values in registers.  Fragment i of a lane then
//     belongs to output row  slot*TM + i  instead of  i*32 + slot.
//   * The MFMA is issued with the operands swapped in NT mode (D = B-frag x A-frag),
//     so in both modes a lane ends up with groups of 4 adjacent output columns; the
//     epilogue packs them to bf16, stages the whole C tile in LDS (the operand
//     stages are dead by then) and writes full rows with 16-byte stores.
// fp32 path (check mode): plain LDS-tiled FMA kernel.
#include <type_traits>

#include "common.h"
#include "mfma_util.h"

namespace cf {

struct GemmArgs {
    const void* A[3];
    const void* B[3];
    int K[3];
    int nseg;
    void* C;
    int M, N;
    float beta;
};

static constexpr int BK = 32;        // K step
static constexpr int STAGES = 4;     // LDS stages (3 K-steps in flight)

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

template <int MODE, int WGM, int WGN, int TM, int TN>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_kernel(GemmArgs g) {
    constexpr int NW = WGM * WGN, NTHREADS = 64 * NW;
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
    constexpr int A_LD = A_BYTES / (1024 * NW), B_LD = B_BYTES / (1024 * NW);   // 1 KB wave-loads per wave per tile
    static_assert(A_LD >= 1 && B_LD >= 1, "tile too small for the wave count");
    constexpr int LD = A_LD + B_LD;
    constexpr unsigned OOB = 0xFFFFFFFFu;
    constexpr int C_PITCH = BN * 2 + 16;                           // staged C tile row pitch (bytes)
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
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

    // ---- global -> LDS: one K-step of both operand tiles -------------------------
    // Wave w, load i fills LDS bytes [(NW*i + w) KB, +1 KB) of the tile; lane l owns
    // the 16 bytes at +16*l.  Offsets are relative to the block's first row / column.
    int seg = 0, k0 = 0, Kseg = 0;       // K-step that the next issue_loads() fetches
    i32x4_t rsA, rsB;
    unsigned ldA = 0, ldB = 0;           // row pitch in bytes of the current segment's operands
    auto open_segment = [&](int s) __attribute__((always_inline)) {
        const bf16_t* A = static_cast<const bf16_t*>(g.A[s]);
        const bf16_t* B = static_cast<const bf16_t*>(g.B[s]);
        Kseg = g.K[s];
        const int64_t K = Kseg;
        if (MODE == 0) {
            rsA = make_rsrc(A + (int64_t)m0 * K, ((int64_t)g.M - m0) * K * 2);
            rsB = make_rsrc(B + (int64_t)n0 * K, ((int64_t)g.N - n0) * K * 2);
            ldA = ldB = (unsigned)K * 2u;
        } else {
            rsA = make_rsrc(A + m0, (K * g.M - m0) * 2);
            rsB = make_rsrc(B + n0, (K * g.N - n0) * 2);
            ldA = (unsigned)g.M * 2u;
            ldB = (unsigned)g.N * 2u;
        }
    };
    auto issue_loads = [&](int stage) __attribute__((always_inline)) {
        const unsigned sa = __builtin_amdgcn_readfirstlane(lds_addr_of(smem) + stage * STAGE + wave * 1024);
        const unsigned sb = sa + A_BYTES;
        if (MODE == 0) {
            // slot = 16 rows x 4 chunks per wave-load; the chunk a lane fetches undoes the XOR swizzle
            const unsigned lc = (lane & 3) ^ ((lane >> 4) & 3);
            const unsigned kb = (k0 + (int)lc * 8 < Kseg) ? (unsigned)(k0 + (int)lc * 8) * 2u : OOB;
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const unsigned row = (NW * i + wave) * 16 + (lane >> 2);
                dma16(sa + i * NW * 1024, rsA, kb == OOB ? OOB : row * ldA + kb);
            }
#pragma unroll
            for (int i = 0; i < B_LD; ++i) {
                const unsigned row = (NW * i + wave) * 16 + (lane >> 2);
                dma16(sb + i * NW * 1024, rsB, kb == OOB ? OOB : row * ldB + kb);
            }
        } else {
            // tile [32][BM] as in memory: a wave-load covers 1024 / (BM*2) k-rows
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const int q = (NW * i + wave) * 64 + lane;
                const int kr = q / (BM / 8), c = q % (BM / 8);
                const bool ok = (m0 + c * 8 < g.M) && (k0 + kr < Kseg);
                dma16(sa + i * NW * 1024, rsA, ok ? (unsigned)(k0 + kr) * ldA + c * 16u : OOB);
            }
#pragma unroll
            for (int i = 0; i < B_LD; ++i) {
                const int q = (NW * i + wave) * 64 + lane;
                const int kr = q / (BN / 8), c = q % (BN / 8);
                const bool ok = (n0 + c * 8 < g.N) && (k0 + kr < Kseg);
                dma16(sb + i * NW * 1024, rsB, ok ? (unsigned)(k0 + kr) * ldB + c * 16u : OOB);
            }
        }
        k0 += BK;
        if (k0 >= Kseg) {
            k0 = 0;
            ++seg;
            if (seg < g.nseg) open_segment(seg);
        }
    };

    // ---- LDS -> MFMA fragments of one 16-wide K sub-step ------------------------
    struct Frags {
        bf16x8_t a[TM], b[TN];
    };
    // NT: tile [rows][32]; the lane reads row row0 + i*32 + slot, logical chunk ks*2 + hh
    const int nt_sw = (slot >> 2) & 3;
    auto frags_nt = [&](const unsigned char* tile, int row0, int ks, bf16x8_t* frag, auto ntiles) __attribute__((always_inline)) {
        constexpr int NT_ = decltype(ntiles)::value;
        const unsigned char* p = tile + (row0 + slot) * 64 + (((ks * 2 + hh) ^ nt_sw) << 4);
#pragma unroll
        for (int i = 0; i < NT_; ++i)
            frag[i] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(p + i * 32 * 64));
    };
    // TN: tile [32][W] as in memory; the lane owns columns col0 + slot*NT_ .. +NT_-1
    auto frags_tn = [&](const unsigned char* tile, int W, int col0, int ks, bf16x8_t* frag, auto ntiles) __attribute__((always_inline)) {
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
    auto load_frags = [&](int stage, int ks, Frags& f) __attribute__((always_inline)) {
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
    // NT: D = Bfrag x Afrag  -> lane = output row (m slot), registers = output columns
    // TN: D = Afrag x Bfrag  -> lane = n slot (TN adjacent columns per lane), registers = m slots
    auto mma = [&](const Frags& f) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = (MODE == 0)
                                ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j], f.a[i], acc[i][j], 0, 0, 0)
                                : __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
    };

    // ---- main loop ------------------------------------------------------------------
    // Iteration t multiplies K-step t out of stage t%4.  At its start the loads of K-step
    // t+3 are issued into the stage that K-step t-1 used (all its reads were issued before
    // the barrier of iteration t-1).  Between the two sub-steps every wave waits until its
    // own loads of K-step t+1 have landed, then the barrier publishes them.
    if (total_steps > 0) {
        Frags f0, f1;
        open_segment(0);
        issue_loads(0);
        if (total_steps > 1) issue_loads(1);
        if (total_steps > 2) issue_loads(2);
        if (total_steps > 2) wait_vmcnt<2 * LD>();
        else if (total_steps > 1) wait_vmcnt<LD>();
        else wait_vmcnt<0>();
        lds_barrier();
        load_frags(0, 0, f0);
        for (int t = 0; t < total_steps; ++t) {
            const int cur = t & (STAGES - 1);
            if (t + 3 < total_steps) issue_loads((t + 3) & (STAGES - 1));
            CF_SCHED_FENCE();
            load_frags(cur, 1, f1);
            CF_SCHED_FENCE();
            mma(f0);
            CF_SCHED_FENCE();
            if (t + 3 < total_steps) wait_vmcnt<2 * LD>();
            else if (t + 2 < total_steps) wait_vmcnt<LD>();
            else wait_vmcnt<0>();
            lds_barrier();
            if (t + 1 < total_steps) load_frags((t + 1) & (STAGES - 1), 0, f0);
            CF_SCHED_FENCE();
            mma(f1);
            CF_SCHED_FENCE();
        }
    }

    // ---- epilogue: acc -> bf16 -> LDS C tile -> global with 16-byte stores -----------
    lds_barrier();      // every wave is done reading operand stages
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                int r, c;     // tile-local row and first column of 4 adjacent outputs
                uint2 o;
                if (MODE == 0) {
                    r = wm * TM * 32 + i * 32 + slot;
                    c = wn * TN * 32 + j * 32 + 8 * v4 + 4 * hh;
                    o.x = pack_bf16x2(acc[i][j][4 * v4 + 0], acc[i][j][4 * v4 + 1]);
                    o.y = pack_bf16x2(acc[i][j][4 * v4 + 2], acc[i][j][4 * v4 + 3]);
                    *reinterpret_cast<uint2*>(smem + r * C_PITCH + c * 2) = o;
                }
            }
        }
    }
    if (MODE == 1) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = wm * TM * 32 + (8 * (v >> 2) + 4 * hh + (v & 3)) * TM + i;
                const int c = wn * TN * 32 + slot * TN;
                if (TN == 4) {
                    uint2 o;
                    o.x = pack_bf16x2(acc[i][0][v], acc[i][1][v]);
                    o.y = pack_bf16x2(acc[i][TN - 2][v], acc[i][TN - 1][v]);
                    *reinterpret_cast<uint2*>(smem + r * C_PITCH + c * 2) = o;
                } else {
                    *reinterpret_cast<unsigned*>(smem + r * C_PITCH + c * 2) = pack_bf16x2(acc[i][0][v], acc[i][1][v]);
                }
            }
        }
    }
    lds_barrier();
    {
        bf16_t* C = static_cast<bf16_t*>(g.C);
        const float beta = g.beta;
        constexpr int CPR = BN / 8;                  // 16-byte chunks per tile row
        constexpr int RPP = NTHREADS / CPR;          // rows per pass
        const int c = tid % CPR, r0 = tid / CPR;
        const int n = n0 + c * 8;
        if (n < g.N) {                                // N is a multiple of 8
#pragma unroll 4
            for (int r = r0; r < BM; r += RPP) {
                const int m = m0 + r;
                if (m >= g.M) break;
                u32x4_t val = *reinterpret_cast<const u32x4_t*>(smem + r * C_PITCH + c * 16);
                bf16_t* p = C + (int64_t)m * g.N + n;
                if (beta != 0.f) {
                    const u32x4_t old = *reinterpret_cast<const u32x4_t*>(p);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(val[e] << 16) + beta * __uint_as_float(old[e] << 16);
                        const float hi = __uint_as_float(val[e] & 0xFFFF0000u) +
                                         beta * __uint_as_float(old[e] & 0xFFFF0000u);
                        val[e] = pack_bf16x2(lo, hi);
                    }
                }
                *reinterpret_cast<u32x4_t*>(p) = val;
            }
        }
    }
}

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;

// per-k-row XOR (in units of 32 bytes) of the K-major tiles: the 8 rows one transpose read
// touches, {4j + r, 8 + 4j + r : r < 4}, land in 8 different 32-byte bank groups
__device__ __forceinline__ int tn_swz(int k) { return (k & 3) | ((k & 8) >> 1); }

// ---------------------------------------------------------------------------
// Large-tile kernel: 256x256 block, 4 waves of 128x128 (the wave tile with the
// fewest LDS bytes per MFMA).  Operand tiles move in K-steps of 32 through a ring
// of five 32 KB LDS stages; the loads of two consecutive K-steps (one whole
// 128-byte line of every operand row) are issued back to back, a full 64-wide
// step ahead of the barrier that publishes them.  The instruction stream is laid
// out by hand: each MFMA is preceded by at most one global->LDS load and one
// fragment read for the following 16-wide sub-step, so no burst of memory
// instructions stands between two MFMAs.  One LDS barrier per 64 MFMAs of a wave.
//   NT stage: [256 rows][32 k], 64-byte rows, 16-byte chunk XOR (row/4)%4.
//   TN stage: [32 k][256 m] as in memory with the chunk index XOR-swizzled per
//   k-row; fragments come out of LDS through the transpose read, in the same
//   register layout as the NT ones, so MFMA order and epilogue are shared.
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void gemm_bf16_ring_kernel(GemmArgs g) {
    constexpr int TM = 4, TN = 4, BM = 256, BN = 256, KB = 32, NST = 5;
    constexpr int A_BYTES = BM * KB * 2, STAGE = 2 * A_BYTES;       // 16 KB + 16 KB
    constexpr int LDH = 8;                                          // wave-loads per wave per K-step
    constexpr unsigned OOB = 0xFFFFFFFFu;
    constexpr int C_PITCH = BN * 2 + 16;
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

    const int total_steps = (g.K[0] + KB - 1) / KB + (g.K[1] + KB - 1) / KB + (g.K[2] + KB - 1) / KB;

    // ---- global -> LDS -----------------------------------------------------------
    // (seg, k0): the K-step that the next load group fetches.  Past the last segment the
    // descriptor of segment 0 stays in place with Kseg = 0, so every load is out of range
    // (zero fill into a stage nobody reads): the number of loads per K-step never changes,
    // which keeps the vmcnt bookkeeping constant.
    int seg = 0, k0 = 0, Kseg = 0;
    i32x4_t rsA, rsB;
    unsigned ldA = 0, ldB = 0;
    auto open_segment = [&](int s) __attribute__((always_inline)) {
        const bool live = s < g.nseg;
        const bf16_t* A = static_cast<const bf16_t*>(s == 1 ? g.A[1] : (s == 2 ? g.A[2] : g.A[0]));
        const bf16_t* B = static_cast<const bf16_t*>(s == 1 ? g.B[1] : (s == 2 ? g.B[2] : g.B[0]));
        const int Kraw = s == 1 ? g.K[1] : (s == 2 ? g.K[2] : g.K[0]);
        Kseg = live ? Kraw : 0;
        const int64_t K = Kraw;
        if (MODE == 0) {
            rsA = make_rsrc(A + (int64_t)m0 * K, ((int64_t)g.M - m0) * K * 2);
            rsB = make_rsrc(B + (int64_t)n0 * K, ((int64_t)g.N - n0) * K * 2);
            ldA = ldB = (unsigned)K * 2u;
        } else {
            rsA = make_rsrc(A + m0, (K * g.M - m0) * 2);
            rsB = make_rsrc(B + n0, (K * g.N - n0) * 2);
            ldA = (unsigned)g.M * 2u;
            ldB = (unsigned)g.N * 2u;
        }
    };
#define CF_ADVANCE_KSTEP()          \
    do {                            \
        k0 += KB;                   \
        if (k0 >= Kseg) {           \
            k0 = 0;                 \
            ++seg;                  \
            open_segment(seg);      \
        }                           \
    } while (0)

    const unsigned lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(smem) + wave * 1024);
    // wave-load u (0..7) of K-step (seg, kk0): u < 4 -> A tile, else B tile; tile bytes [(4*(u%4) + wave) KB, +1 KB)
    // NT: 16 rows x 4 chunks, the chunk a lane fetches undoes the XOR swizzle of its LDS slot
    // TN: 2 k-rows x 32 chunks
    const unsigned nt_lc = (unsigned)((lane & 3) ^ ((lane >> 4) & 3));
    auto dma_one = [&](int stage, int u, int kk0) __attribute__((always_inline)) {
        const bool isA = u < 4;
        const int i = u & 3;
        const unsigned dst = lds0 + stage * STAGE + (isA ? 0 : A_BYTES) + i * 4096;
        unsigned off;
        if (MODE == 0) {
            const unsigned row = (4 * i + wave) * 16 + (lane >> 2);
            const int kk = kk0 + (int)nt_lc * 8;
            off = (kk < Kseg) ? row * (isA ? ldA : ldB) + (unsigned)kk * 2u : OOB;
        } else {
            const int qq = (4 * i + wave) * 64 + lane;
            const int kr = qq >> 5;
            const int c = (qq & 31) ^ (tn_swz(kr) << 1);
            const bool ok = ((isA ? m0 : n0) + c * 8 < (isA ? g.M : g.N)) && (kk0 + kr < Kseg);
            off = ok ? (unsigned)(kk0 + kr) * (isA ? ldA : ldB) + c * 16u : OOB;
        }
        if (isA) dma16(dst, rsA, off);
        else dma16(dst, rsB, off);
    };

    // ---- LDS -> fragments ------------------------------------------------------------
    bf16x8_t fa[2][TM], fb[2][TN];
    const int nt_sw = (slot >> 2) & 3;
    auto frag_one = [&](int stage, int ks, int u, int buf) __attribute__((always_inline)) {
        const bool isA = u < 4;
        const int i = u & 3;
        const unsigned char* tile = smem + stage * STAGE + (isA ? 0 : A_BYTES);
        bf16x8_t f;
        if (MODE == 0) {
            const int row = (isA ? wm : wn) * 128 + i * 32 + slot;
            f = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(
                                                 tile + row * 64 + (((ks * 2 + hh) ^ nt_sw) << 4)));
        } else {
            const int k = ks * 16 + 8 * hh + ((lane & 15) >> 2);
            const int lc = ((isA ? wm : wn) * 128 + i * 32) / 8 + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
            const int sub = (lane & 1) * 8;
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_s16x4_ptr)(tile + k * 512 + ((lc ^ (tn_swz(k) << 1)) << 4) + sub));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (lds_s16x4_ptr)(tile + (k + 4) * 512 + ((lc ^ (tn_swz(k + 4) << 1)) << 4) + sub));
            f = __builtin_bit_cast(bf16x8_t, (s16x8_t)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
        if (isA) fa[buf][i] = f;
        else fb[buf][i] = f;
    };
    // MFMA q (0..15) of a sub-step: D = Bfrag x Afrag, lane = output row, registers = 4-column groups
    auto mma_one = [&](int q, int buf) __attribute__((always_inline)) {
        const int i = q >> 2, j = q & 3;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
    };
    // one 16-wide sub-step: MFMAs on fragment buffer `buf`; the fragments of (stage ns, sub-step nks)
    // go into the other buffer; with_dma: the 16 loads of the next two K-steps, one per MFMA,
    // the two halves of each 128-byte line adjacent
    auto substep = [&](int buf, int ns, int nks, bool with_dma, int st0, int st1) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            if (with_dma) {
                if ((q & 1) == 0) dma_one(st0, q >> 1, k0);
                else dma_one(st1, q >> 1, k0 + KB);
            }
            if ((q & 1) == 0) frag_one(ns, nks, q >> 1, buf ^ 1);
            CF_SCHED_FENCE();
            mma_one(q, buf);
            CF_SCHED_FENCE();
        }
    };
    // loads of two consecutive K-steps outside the MFMA stream (prologue)
    auto issue_pair = [&](int st0, int st1) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            dma_one(st0, u, k0);
            dma_one(st1, u, k0 + KB);
        }
    };
    // A pair never straddles a segment boundary unless the segment's K is not a multiple of 64;
    // then the second half reads past Kseg and is zero-filled, and the next pair restarts at
    // the new segment (see advance below): K-steps are counted per segment in units of 32, and
    // a segment with an odd count gets one all-zero K-step appended.
#define CF_ADVANCE_PAIR()            \
    do {                             \
        k0 += 2 * KB;                \
        if (k0 >= Kseg) {            \
            k0 = 0;                  \
            ++seg;                   \
            open_segment(seg);       \
        }                            \
    } while (0)

    // number of K-steps of 32 including the zero padding of odd segments
    const int steps = 2 * ((g.K[0] + 2 * KB - 1) / (2 * KB) + (g.K[1] + 2 * KB - 1) / (2 * KB) +
                           (g.K[2] + 2 * KB - 1) / (2 * KB));
    (void)total_steps;

    if (steps > 0) {
        open_segment(0);
        issue_pair(0, 1);
        CF_ADVANCE_PAIR();
        issue_pair(2, 3);
        CF_ADVANCE_PAIR();
        wait_vmcnt<2 * LDH>();          // K-steps 0 and 1 have landed; 2 and 3 may be in flight
        lds_barrier();
#pragma unroll
        for (int u = 0; u < 8; ++u) frag_one(0, 0, u, 0);
        int st = 0;                     // stage of the current K-step
        for (int s = 0; s < steps; s += 2) {
            // ---- even K-step s (stage st): no loads, no barrier: K-step s+1 was published
            //      together with K-step s at the barrier of the previous pair
            const int st1 = st + 1 >= NST ? st + 1 - NST : st + 1;
            substep(0, st, 1, false, 0, 0);
            substep(1, st1, 0, false, 0, 0);
            // ---- odd K-step s+1 (stage st1) ----------------------------------------------
            const int st2 = st1 + 1 >= NST ? st1 + 1 - NST : st1 + 1;
            const int st3 = st2 + 2 >= NST ? st2 + 2 - NST : st2 + 2;  // (s+4) % 5
            substep(0, st1, 1, false, 0, 0);
            wait_vmcnt<0>();            // K-steps s+2, s+3 have landed (nothing else is in flight)
            lds_barrier();              // ... and every wave is done with stages st and (s+4)%5
            substep(1, st2, 0, true, st3, st);      // loads of K-steps s+4 -> st3, s+5 -> st
            CF_ADVANCE_PAIR();
            st = st2;
        }
        wait_vmcnt<0>();
    }
#undef CF_ADVANCE_KSTEP
#undef CF_ADVANCE_PAIR

    // ---- epilogue: acc -> bf16 -> LDS C tile -> global with 16-byte stores -----------
    lds_barrier();
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const int r = wm * 128 + i * 32 + slot;
                const int c = wn * 128 + j * 32 + 8 * v4 + 4 * hh;
                uint2 o;
                o.x = pack_bf16x2(acc[i][j][4 * v4 + 0], acc[i][j][4 * v4 + 1]);
                o.y = pack_bf16x2(acc[i][j][4 * v4 + 2], acc[i][j][4 * v4 + 3]);
                *reinterpret_cast<uint2*>(smem + r * C_PITCH + c * 2) = o;
            }
    lds_barrier();
    {
        bf16_t* C = static_cast<bf16_t*>(g.C);
        const float beta = g.beta;
        const int c = tid & 31, r0 = tid >> 5;
        const int n = n0 + c * 8;
        if (n < g.N) {
#pragma unroll 4
            for (int r = r0; r < BM; r += 8) {
                const int m = m0 + r;
                if (m >= g.M) break;
                u32x4_t val = *reinterpret_cast<const u32x4_t*>(smem + r * C_PITCH + c * 16);
                bf16_t* p = C + (int64_t)m * g.N + n;
                if (beta != 0.f) {
                    const u32x4_t old = *reinterpret_cast<const u32x4_t*>(p);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(val[e] << 16) + beta * __uint_as_float(old[e] << 16);
                        const float hi = __uint_as_float(val[e] & 0xFFFF0000u) +
                                         beta * __uint_as_float(old[e] & 0xFFFF0000u);
                        val[e] = pack_bf16x2(lo, hi);
                    }
                }
                *reinterpret_cast<u32x4_t*>(p) = val;
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

template <int MODE>
static hipError_t launch_ring(const GemmArgs& g, hipStream_t st) {
    constexpr int smem = 5 * 32768;                 // five operand stages; the C tile staging (132 KB) reuses them
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_ring_kernel<MODE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int grid = ceil_div(g.M, 256) * ceil_div(g.N, 256);
    gemm_bf16_ring_kernel<MODE><<<grid, 256, smem, st>>>(g);
    return hipGetLastError();
}

template <int MODE, int WGM, int WGN, int TM, int TN>
static hipError_t launch_bf16(const GemmArgs& g, hipStream_t st) {
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    constexpr int stages = STAGES * (BM + BN) * BK * 2;
    constexpr int ctile = BM * (BN * 2 + 16);
    constexpr int smem = stages > ctile ? stages : ctile;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<MODE, WGM, WGN, TM, TN>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int grid = ceil_div(g.M, BM) * ceil_div(g.N, BN);
    gemm_bf16_kernel<MODE, WGM, WGN, TM, TN><<<grid, 64 * WGM * WGN, smem, st>>>(g);
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
    // big: 256x256 block, 8 waves (2 per SIMD) of 128x64; small: 128x128 block, 4 waves of 64x64
    if (big) return mode == 0 ? launch_ring<0>(g, st) : launch_ring<1>(g, st);
    if (mode == 0) return big ? launch_bf16<0, 2, 4, 4, 2>(g, st) : launch_bf16<0, 2, 2, 2, 2>(g, st);
    return big ? launch_bf16<1, 2, 4, 4, 2>(g, st) : launch_bf16<1, 2, 2, 2, 2>(g, st);
}

}  // namespace cf
