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
// bf16 path: 16x16x32 bf16 MFMA, fp32 accumulators, 256 threads = 2x2 waves, one
// block per CU.  The block tile is (64*TM) x (64*TN) with wave tiles of
// (32*TM) x (32*TN); three shapes are compiled into one kernel: 256x256 (the
// wave tile with the fewest LDS bytes per MFMA), 256x128 and 128x128; the NT kernel
// also has 256x192, for outputs whose 256x256 tiles would leave CUs idle (a dX of
// 4096 x 3072 is 16 x 12 = 192 such tiles but 16 x 16 = 256 of the narrower ones).
//   * Why the small MFMA.  Under these kernels the chip is power-limited: the shader clock
//     settles at 1.5-1.9 GHz instead of 2.4, and 128 CUs deliver 75 % of what 256 do.
//     What counts is therefore energy per flop, not only cycles: 16x16x32 reads and writes
//     its accumulators half as often per flop as 32x32x16 does, runs at a 14 % higher
//     clock for the same work and gains 3-6 % on the large products, although its
//     16-cycle issue rhythm leaves less room for the other instructions (the matrix
//     cores are busy 72 % of the cycles instead of 77 %).  Fragment reads from LDS cost
//     no cycles any more but about 9 % of the clock.
//   * Tile scheduling.  A launch has as many blocks as CUs; a block walks through its
//     share of the output tiles.  The 256x256 tiles that fill whole rounds of the CUs
//     come first; the tiles of the last, partial round are cut into 2 or 4 sub-tiles
//     when that shortens the tail (a 3.5-round problem takes 3 rounds of full tiles
//     and one of half tiles instead of 4 rounds).  Within each group the 8 XCDs (block
//     id mod 8) take contiguous runs of a band-major tile order, so the blocks resident
//     on one XCD share operand panels in that XCD's L2.  Between two tiles of a block
//     the loads of the next tile's first K-steps are already in flight while the
//     finished tile leaves, and its stores drain under the next tile's MFMAs (the
//     write-out of a tile used to be 13 % of its time).
//   * Operand tiles move in K-steps of 32 through a ring of four 32 KB LDS stages,
//     filled by buffer_load ... lds (16 bytes per lane, no register hop).  K-steps are
//     handled in pairs (64 k: one whole 128-byte line of every NT operand row, fetched
//     by two adjacent instructions); a pair is loaded two pairs ahead, into the two
//     stages that the barrier of the pair being computed has just retired; completion
//     is tracked with vmcnt.  Ragged edges come from the buffer descriptor's range
//     check, which returns zeros, so there are no branches around loads.
//   * One LDS barrier per 64 K.  A pair is 2*TM sub-steps: one 32-row block of the
//     wave's A rows against all its B columns for one K-step (16 MFMAs in a 128x128 wave
//     tile).  The A fragments of the next sub-step and a share of the B fragments of
//     the next K-step are read ahead of their use, and the instruction stream is laid
//     out by hand: a gap between two MFMAs carries at most one fragment read and one
//     instruction of a load (the write of M0 goes ahead of an MFMA, the load behind it).
//     The loop body is two pairs, which makes every stage a compile-time constant: an
//     LDS read is a loop-invariant per-lane base register plus an instruction offset, a
//     load takes its per-lane offset from a register that is fixed for the whole K
//     segment and its K position from the instruction's scalar offset, so the steady
//     state has no vector ALU instruction besides the MFMAs.
//   * The loads of a pair go out in groups spread over the sub-steps (four groups in
//     NT, three in TN; two cost 4 %): a CU sustains only so many bytes in flight, and a
//     burst of 64 KB stalls the stream.
//   * NT stage: [rows][32 k], 64-byte rows, the 16-byte chunk index of a row XOR-ed with a
//     function of row/4 chosen so that the 16 lanes that the LDS serves in one pass of a
//     ds_read_b128 hit distinct banks (see nt_swz); a lane of the loading wave picks the
//     global chunk that belongs in its (fixed) LDS slot.
//   * TN stage: [32 k][rows] exactly as in memory, with the 64-byte group index of a
//     k-row XOR-ed with k%4; fragments come out of LDS through the transpose read
//     (ds_read_b64_tr_b16), in the same register layout as the NT ones, so MFMA
//     order and epilogue are shared.  The four k-rows that a group of 16 lanes touches
//     in one transpose read land in four different 64-byte bank groups.
//   * The MFMA is issued with the operands swapped (D = B-frag x A-frag), so a lane
//     ends up with 4 adjacent output columns of one row; the epilogue packs them to
//     bf16 and sends them, 32 rows of the wave tile at a time, through 8 KB of LDS of
//     the wave's own (above the operand stages, which the next tile is filling by
//     then) to full-row 16-byte stores.
// fp32 path (check mode): plain LDS-tiled FMA kernel.
#include <algorithm>
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
    float alpha;    // the product is scaled by alpha before beta*C is added
    int c_f32;      // bf16 kernels: C is fp32 (a main-gradient buffer), written without rounding
    int n_full;     // leading blocks that own a whole 256x256 tile
    int sub;        // the remaining tiles are cut into `sub` (1, 2 or 4) sub-tiles, one block each
    int tile_n;     // 256, or 192 (NT, bf16 output only): every tile is 256x192 and n_full, sub are unused
    // Column groups (ngroups > 1, one K segment): output columns [off_j, off_j + Ng[j]) belong to a
    // matrix of their own, C = Cg[j] [M, Ng[j]] with B operand Bg[j]; every Ng[j] is a multiple of
    // 256, so a tile lies in one group.  N is the sum of the Ng.  One launch then covers several
    // products that share their A operand (the dW of the q, k and v projections).
    int ngroups;
    const void* Bg[3];
    void* Cg[3];
    int Ng[3];
    // Kept-token count on the device (nullable).  When set, the kept-token dimension handed in by the
    // host (M in mode NT, K[0] in mode TN) is only an upper bound: every block reads the count, takes
    // min(count, bound) for that dimension and, in mode NT, plans the tiles itself (plan_launch).
    const int32_t* n_dev;
    // Mode NT, segment 0 (nullable): row m of A is row a_idx[m] of a matrix with a_rows rows (the
    // gather of the upstream gradient's kept rows, folded into the A-tile loads).
    const int32_t* a_idx;
    int64_t a_rows;
};

// How the tiles of the last, partial round are cut.  The cost of a round of sub-tiles
// relative to a round of 256x256 tiles is more than its share of the flops (smaller
// tiles move more operand bytes per flop); the figures are measured on MI355X at K = 4096.
// Returns the launch's length in rounds of 256x256 tiles.
// A round of 256x192 tiles costs 0.94 of a round of 256x256 tiles although it has 0.75 of the
// flops: the chip is power-limited under these kernels, so the 192 CUs that a 16 x 12 tile output
// occupies clock higher than all 256 do (measured: 412 GFLOP in 354 us on 192 CUs, 333 us on 256).
static constexpr double kCost192 = 0.94;
__host__ __device__ inline int cdiv(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline double plan_tiles(int tiles, int n_cu, int& n_full, int& sub) {
    n_full = tiles / n_cu * n_cu;
    const int rem = tiles - n_full;
    sub = 1;
    if (rem == 0) return n_full / n_cu;
    double best = 1e30;
    for (int c = 0; c < 3; ++c) {
        const double cost = c == 0 ? 1.0 : (c == 1 ? 0.6 : 0.4);
        const int cut = 1 << c;
        const double t = (double)cdiv(rem * cut, n_cu) * cost;
        if (t < best - 1e-9) {
            best = t;
            sub = cut;
        }
    }
    return n_full / n_cu + best;
}

// Tile plan of a bf16 launch with n_cu blocks: sets n_full, sub, tile_n; returns the number of work
// items.  The host plans a launch whose sizes it knows; with a device-side count every block runs
// the same code on the count it read, so both give the same tiles for the same sizes.
__host__ __device__ inline int plan_launch(int M, int N, int mode, bool c_f32, int ngroups, int n_cu,
                                           int& n_full, int& sub, int& tile_n) {
    const int tiles = cdiv(M, 256) * cdiv(N, 256);
    const double rounds = plan_tiles(tiles, n_cu, n_full, sub);
    int items = n_full + (tiles - n_full) * sub;
    tile_n = 256;
    if (mode == 0 && !c_f32 && ngroups == 1) {
        // 256x192 tiles instead, when they fill the CUs better (an output of 16 x 12 tiles of
        // 256x256 leaves a quarter of the CUs idle; as 16 x 16 tiles of 256x192 it is one full round)
        const int tiles192 = cdiv(M, 256) * cdiv(N, 192);
        if (cdiv(tiles192, n_cu) * kCost192 < rounds - 1e-9) {
            tile_n = 192;
            items = tiles192;
        }
    }
    return items;
}

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;

static constexpr int GEMM_STAGES = 4;
static constexpr int GEMM_STAGE_BYTES = 32768;
static constexpr int GEMM_SMEM = 160 * 1024;    // the whole LDS of a CU: four operand stages; the C tile staging of the epilogue needs 132 KB

// Position l of a block in the logical order of its group of n blocks: XCD x (block id
// mod 8) takes the x-th contiguous share of the order.
__device__ __forceinline__ int xcd_order(int pid, int n) {
    const int xcd = pid & 7, local = pid >> 3;
    const int base = n >> 3, rem = n & 7;
    return xcd * base + (xcd < rem ? xcd : rem) + local;
}

// Logical tile l -> tile coordinates: bands of GROUP_M tile rows walked column by column.
__device__ __forceinline__ void tile_coords(int l, int tiles_m, int tiles_n, int& bm, int& bn) {
    constexpr int GROUP_M = 8;
    const int band = l / (GROUP_M * tiles_n);
    const int first_m = band * GROUP_M;
    const int gsize = min(GROUP_M, tiles_m - first_m);
    const int r = l - band * GROUP_M * tiles_n;
    bm = first_m + r % gsize;
    bn = r / gsize;
}

template <typename P>
__device__ __forceinline__ P* uniform_ptr(P* p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<P*>(((uint64_t)hi << 32) | lo);
}

// Swizzle of an NT stage: the 16-byte chunk index of row r is XOR-ed with nt_swz(r / 4) = {0, 2, 3, 1}
// [(r / 4) % 4].  The LDS serves a ds_read_b128 in four passes of 16 lanes, and the passes are not
// runs of consecutive lanes: {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31} and the same plus 32
// (measured).  A fragment read has lane l at row l % 16, chunk l / 16, so a pass mixes chunk c of rows
// 0-3 and 12-15 with chunk c + 1 of rows 4-11 (or the other way round); with this table the 16
// lanes of every pass fall into 16 different 16-byte bank groups (with r / 4 itself they do not).
__device__ __forceinline__ int nt_swz(int q) { return (0x78 >> (2 * (q & 3))) & 3; }

// Of D loads spread over the N MFMAs of a sub-step (D <= N), the one that goes with MFMA q, or -1.
constexpr int load_in_gap(int q, int D, int N) {
    for (int d = 0; d < D; ++d)
        if ((d * N) / D == q) return d;
    return -1;
}

// One output tile: its origin, and the B operand (of segment 0), output matrix and column count
// it belongs to (those of its column group in a grouped launch).
struct TileRef {
    int m0, n0, N;
    const void* B0;
    void* C;
};

// The block's output tiles of (64*TM) x (64*TN), one after the other: `first`, then whatever
// next_tile(TileRef&) hands out until it returns false.  With bf16 output the loads of the next
// tile's first K-steps are in flight while the finished tile leaves through a staging area of its
// own, and its stores drain under the next tile's MFMAs.  SPLIT: the block contracts only k in
// [kbeg, kend) of the single segment and stores its fp32 accumulators, unscaled, to `part_out`
// ([M, N] fp32); a second kernel adds the parts up.
// Mx, K0x: the live values of g.M and g.K[0] (they differ from the launch arguments when the
// kept-token count is read on the device).
template <int MODE, int TM, int TN, bool SPLIT, bool CF32, typename Next>
__device__ __forceinline__ void gemm_tiles(const GemmArgs& g, const int Mx, const int K0x, const TileRef first,
                                           Next next_tile, unsigned char* smem,
                                           const int kbeg = 0, const int kend = 0, float* part_out = nullptr) {
    constexpr int BM = 64 * TM, BN = 64 * TN, KB = 32, STAGE = GEMM_STAGE_BYTES;
    constexpr int A_BYTES = BM * KB * 2;                // B tile follows the A tile inside a stage
    constexpr int NU = TM + TN;                         // 1 KB wave-loads per wave per K-step: TM for A, TN for B
    constexpr int FM = 2 * TM, FN = 2 * TN;             // 16-row fragments of the wave tile along M and N
    constexpr int NQ = 2 * FN;                          // MFMAs per sub-step: one 32-row block of A x all of B
    // groups that the wave-loads of a pair are issued in (measured: 2 groups cost 4 %; NT is best
    // with 4 to 6, TN with 3)
    constexpr int NG = TM == 2 ? 2 : (MODE == 0 ? 4 : 3);
    static_assert(A_BYTES + BN * KB * 2 <= STAGE, "tile shape");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, g4 = lane >> 4;

    f32x4_t acc[FM][FN];
    TileRef ld = first;             // the tile whose operands are being loaded

    // ---- global -> LDS -----------------------------------------------------------
    // (seg, k0): the K-step that the next loads fetch.  Past the last segment Kseg = 0, so
    // every load is out of range (zero fill into a stage whose contents are never used):
    // the number of loads per K-step never changes, which keeps the vmcnt bookkeeping constant.
    int seg = 0, k0 = 0, Kseg = 0;
    i32x4_t rsA, rsB;
    unsigned ldA = 0, ldB = 0;
    // Per-lane byte offset of wave-load u at k = 0 of the current segment (out of range for rows /
    // columns beyond the matrix edge); the K position of a K-step is added as the load's scalar
    // offset, so the steady-state loop spends no vector instruction on addresses.  v0 / v1 are the
    // offsets used for the first / second K-step of the pair at (seg, k0): equal to vbase while the
    // pair lies inside the segment, out of range for the lanes whose k falls past its end.
    constexpr unsigned OOB_FAST = 0x80000000u;          // stays out of range when the scalar offset is added
    unsigned vbase[NU], v0[NU], v1[NU];
    bool pair_inside = false;
    const unsigned nt_lc = (unsigned)((lane & 3) ^ nt_swz(lane >> 4));
    auto open_segment = [&](int s) __attribute__((always_inline)) {
        const bool live = s < g.nseg;
        const int m0 = ld.m0, n0 = ld.n0;
        const bf16_t* A = static_cast<const bf16_t*>(s == 1 ? g.A[1] : (s == 2 ? g.A[2] : g.A[0]));
        const bf16_t* B = static_cast<const bf16_t*>(s == 1 ? g.B[1] : (s == 2 ? g.B[2] : ld.B0));
        const int Kraw = s == 1 ? g.K[1] : (s == 2 ? g.K[2] : K0x);
        Kseg = live ? Kraw : 0;
        const int64_t K = Kraw;
        const bool gatherA = MODE == 0 && s == 0 && g.a_idx != nullptr;
        if (MODE == 0) {
            // gathered A: the descriptor spans the whole source matrix and a lane's offset starts at its source row
            rsA = gatherA ? make_rsrc(A, g.a_rows * K * 2) : make_rsrc(A + (int64_t)m0 * K, ((int64_t)Mx - m0) * K * 2);
            rsB = make_rsrc(B + (int64_t)n0 * K, ((int64_t)ld.N - n0) * K * 2);
            ldA = ldB = (unsigned)K * 2u;
        } else {
            rsA = make_rsrc(A + m0, (K * Mx - m0) * 2);
            rsB = make_rsrc(B + n0, (K * ld.N - n0) * 2);
            ldA = (unsigned)Mx * 2u;
            ldB = (unsigned)ld.N * 2u;
        }
        // The per-lane parts below never change, but they are cheap to rebuild and registers are
        // scarce while a finished tile is still in the accumulators: keep the compiler from carrying
        // them across the main loop (and spilling them) by hiding where the lane number comes from.
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const unsigned lc_nt = (unsigned)((ln & 3) ^ nt_swz(ln >> 4));
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const bool isA = u < TM;
            const int i = isA ? u : u - TM;
            if (MODE == 0) {
                const unsigned row = (4 * i + wave) * 16 + (ln >> 2);
                vbase[u] = row * (isA ? ldA : ldB) + lc_nt * 16u;
                if (isA && gatherA) {       // rows past M carry an out-of-range offset; the index is read for live rows only
                    const int m = m0 + (int)row;
                    vbase[u] = m < Mx ? (unsigned)g.a_idx[m] * ldA + lc_nt * 16u : OOB_FAST;
                }
            } else {
                const int cpr = (isA ? BM : BN) / 8;
                const int qq = (4 * i + wave) * 64 + ln;
                const int kr = qq / cpr;
                const int c = (qq % cpr) ^ ((kr & 3) << 2);
                const bool ok = (isA ? m0 : n0) + c * 8 < (isA ? Mx : ld.N);
                vbase[u] = ok ? (unsigned)kr * (isA ? ldA : ldB) + c * 16u : OOB_FAST;
            }
        }
        pair_inside = false;
    };
    // offsets and scalar K offsets of the pair at (seg, k0); cheap when this pair and the previous one
    // lie inside the segment
    unsigned ka0 = 0, kb0 = 0, ka1 = 0, kb1 = 0;
    auto prepare_pair = [&]() __attribute__((always_inline)) {
        const bool inside = k0 + 2 * KB <= Kseg;
        if (!(inside && pair_inside)) {
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                int kpos;                       // first k of the lane's chunk within a K-step
                if (MODE == 0) {
                    kpos = (int)nt_lc * 8;
                } else {
                    const bool isA = u < TM;
                    const int i = isA ? u : u - TM;
                    kpos = ((4 * i + wave) * 64 + lane) / ((isA ? BM : BN) / 8);
                }
                v0[u] = (k0 + kpos < Kseg) ? vbase[u] : OOB_FAST;
                v1[u] = (k0 + KB + kpos < Kseg) ? vbase[u] : OOB_FAST;
            }
        }
        pair_inside = inside;
        if (MODE == 0) {
            ka0 = kb0 = (unsigned)k0 * 2u;
            ka1 = kb1 = (unsigned)(k0 + KB) * 2u;
        } else {
            ka0 = (unsigned)k0 * ldA; kb0 = (unsigned)k0 * ldB;
            ka1 = (unsigned)(k0 + KB) * ldA; kb1 = (unsigned)(k0 + KB) * ldB;
        }
    };
    // A pair of K-steps never straddles a segment boundary: a segment with an odd number of
    // K-steps gets one all-zero K-step appended (its loads fall past Kseg).
    auto advance_pair = [&]() __attribute__((always_inline)) {
        k0 += 2 * KB;
        if (k0 >= Kseg) {
            k0 = 0;
            ++seg;
            open_segment(seg);
        }
    };

    const unsigned lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(smem) + wave * 1024);
    // wave-load U of K-step SEC (0 / 1) of the pair at (seg, k0) into stage S: U < TM -> A tile, else B
    // tile; tile bytes [(4*i + wave) KB, +1 KB).  NT: 16 rows x 4 chunks, the chunk a lane fetches undoes
    // the XOR swizzle of its LDS slot; the second K-step of a pair is the other half of the same
    // 128-byte lines (instruction offset 64).  TN: 1024 / (2*rows) k-rows of the tile.
    auto dma_one = [&](auto S, auto U, auto SEC) __attribute__((always_inline)) {
        constexpr int s = decltype(S)::value, u = decltype(U)::value, sec = decltype(SEC)::value;
        constexpr bool isA = u < TM;
        constexpr int i = isA ? u : u - TM;
        constexpr int dst = s * STAGE + (isA ? 0 : A_BYTES) + i * 4096;
        // the instruction offset moves the LDS destination along with the global address, so the
        // M0 base of the second K-step is set back by the same amount
        if (MODE == 0) dma16i<dst - (sec ? KB * 2 : 0), sec ? KB * 2 : 0>(lds0, isA ? rsA : rsB, sec ? v1[u] : v0[u], ka0);
        else dma16i<dst, 0>(lds0, isA ? rsA : rsB, sec ? v1[u] : v0[u], isA ? (sec ? ka1 : ka0) : (sec ? kb1 : kb0));
    };
    // the same load wrapped around the MFMA acc += a x b (inside the MFMA stream)
    auto mma_dma_one = [&](f32x4_t& c, const bf16x8_t a, const bf16x8_t b, auto S, auto U, auto SEC) __attribute__((always_inline)) {
        constexpr int s = decltype(S)::value, u = decltype(U)::value, sec = decltype(SEC)::value;
        constexpr bool isA = u < TM;
        constexpr int i = isA ? u : u - TM;
        constexpr int dst = s * STAGE + (isA ? 0 : A_BYTES) + i * 4096;
        if (MODE == 0)
            mfma16_dma16i<dst - (sec ? KB * 2 : 0), sec ? KB * 2 : 0>(c, a, b, lds0, isA ? rsA : rsB, sec ? v1[u] : v0[u], ka0);
        else
            mfma16_dma16i<dst, 0>(c, a, b, lds0, isA ? rsA : rsB, sec ? v1[u] : v0[u],
                                  isA ? (sec ? ka1 : ka0) : (sec ? kb1 : kb0));
    };

    // ---- LDS -> fragments.  A fragment is 16 rows x 32 k (one K-step): lane l holds row l%16,
    // k = 8*(l/16) .. +7.  An LDS address is a per-lane base register that never changes plus a
    // compile-time constant (stage, fragment) in the instruction's 16-bit offset field; stages 2
    // and 3 lie past that field's reach from the base of stage 0 and get base registers of their own.
    typedef __attribute__((address_space(3))) unsigned char* lds_u8_ptr;
    typedef const __attribute__((address_space(3))) u32x4_t* lds_u32x4_cptr;
    constexpr int NBASE = MODE == 0 ? 2 : NU;       // NT: A, B; TN: one per 32-row block (the swizzle mixes the block in)
    unsigned fbase[NBASE][2];
    {
        const unsigned s0 = lds_addr_of(smem);
        if (MODE == 0) {
            const int nt_sw = nt_swz(l16 >> 2);
#pragma unroll
            for (int ab = 0; ab < 2; ++ab) {
                const int wrow = ab == 0 ? wm * (32 * TM) : wn * (32 * TN);
                const unsigned v = s0 + (ab == 0 ? 0 : A_BYTES) + (wrow + l16) * 64 + ((g4 ^ nt_sw) << 4);
                fbase[ab][0] = v;
                fbase[ab][1] = v + 2 * STAGE;
            }
        } else {
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const bool isA = u < TM;
                const int i = isA ? u : u - TM;
                const int W2 = (isA ? BM : BN) * 2;                 // bytes per k-row
                const int row0 = isA ? wm * (32 * TM) + i * 32 : wn * (32 * TN) + i * 32;
                const int kl = 8 * g4 + (l16 >> 2);                 // k within the K-step (and kl + 4)
                const int lc = row0 / 8 + ((lane & 3) >> 1);
                const int sw = (kl & 3) << 2;                       // the same for k and k + 4
                const unsigned v = s0 + (isA ? 0 : A_BYTES) + kl * W2 + ((lc ^ sw) << 4) + (lane & 1) * 8;
                fbase[u][0] = v;
                fbase[u][1] = v + 2 * STAGE;
            }
        }
    }
    bf16x8_t fa[2][2], fb[2][FN];
    // fragment F (16 rows; F < FM: of the wave's A rows, else of its B rows) of the K-step in stage S
    // into fa[BUF][F % 2] or fb[BUF][F - FM]
    auto frag_one = [&](auto S, auto F, auto BUF) __attribute__((always_inline)) {
        constexpr int s = decltype(S)::value, fr = decltype(F)::value, buf = decltype(BUF)::value;
        constexpr bool isA = fr < FM;
        constexpr int f = isA ? fr : fr - FM;
        constexpr int win = s >> 1, soff = (s & 1) * STAGE;
        bf16x8_t v;
        if (MODE == 0) {
            const lds_u8_ptr p = reinterpret_cast<lds_u8_ptr>(fbase[isA ? 0 : 1][win]);
            v = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<lds_u32x4_cptr>(p + (soff + f * 1024)));
        } else {
            constexpr int W2 = (isA ? BM : BN) * 2;
            const lds_u8_ptr p = reinterpret_cast<lds_u8_ptr>(fbase[(isA ? 0 : TM) + f / 2][win]);
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + (soff + (f & 1) * 32)));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + (soff + (f & 1) * 32 + 4 * W2)));
            v = __builtin_bit_cast(bf16x8_t, (s16x8_t)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
        if constexpr (isA) fa[buf][f & 1] = v;
        else fb[buf][f] = v;
    };
    // Sub-step T of a pair (T = KS*TM + A): the MFMAs of K-step KS (stage ST + KS) for the 32-row
    // block A of the wave's rows against all its columns.  D = Bfrag x Afrag: lane l holds row l%16 of
    // the fragment and 4 adjacent output columns.  Spread between the MFMAs:
    //   * the two A fragments of the next sub-step (the next block of the same K-step, or block 0 of
    //     the next K-step);
    //   * the B fragments of the next K-step: during K-step 0 of the pair a share of those of K-step 1
    //     per sub-step; K-step 0 of the next pair is published by the barrier ahead of the pair's last
    //     sub-step, which therefore reads all of them;
    //   * a share of the wave-loads: the pair at (seg, k0) is loaded in NG groups, group 0 in the last
    //     sub-step of a pair (into the two stages its barrier has just retired), groups 1.. in the first
    //     sub-steps of the next pair, the two halves of each 128-byte line of an NT operand row in
    //     adjacent instructions.
    auto substep = [&](auto ST, auto T) __attribute__((always_inline)) {
        constexpr int st = decltype(ST)::value, t = decltype(T)::value;
        constexpr int ks = t / TM, a = t % TM;
        constexpr int st1 = st + 1, st2 = (st + 2) & 3;
        constexpr bool last = t == 2 * TM - 1;
        constexpr int cur = st + ks;                                // stage of this K-step
        constexpr int nxt = ks == 0 ? st1 : st2;                    // stage of the next K-step
        constexpr int a_stage = a + 1 < TM ? cur : nxt, a_blk = a + 1 < TM ? a + 1 : 0;
        // reads of this sub-step, in the order their first users come: A fragment 0, B fragments, A fragment 1
        constexpr int NB = ks == 0 ? 0 : (last ? FN : 0);           // all B fragments at once
        constexpr int b_lo = ks == 0 ? (a * FN) / TM : 0, b_hi = ks == 0 ? ((a + 1) * FN) / TM : NB;
        constexpr int NR = 2 + (b_hi - b_lo);
        // wave-loads of this sub-step: group 0 (last sub-step) or group t + 1 (t < TM - 1)
        constexpr int grp = last ? 0 : (t < NG - 1 ? t + 1 : -1);
        constexpr int e_lo = grp < 0 ? 0 : ((grp * NU) / NG) * 2, e_hi = grp < 0 ? 0 : (((grp + 1) * NU) / NG) * 2;
        constexpr int d0 = last ? st : st2, d1 = d0 + 1;
        static_for<NQ>([&](auto Q) __attribute__((always_inline)) {
            constexpr int q = decltype(Q)::value;
            static_for<NR>([&](auto R) __attribute__((always_inline)) {
                constexpr int r = decltype(R)::value;
                if constexpr ((r * NQ) / NR == q) {
                    if constexpr (r == 0) frag_one(ic<a_stage>{}, ic<2 * a_blk>{}, ic<((a + 1) & 1)>{});
                    else if constexpr (r == NR - 1) frag_one(ic<a_stage>{}, ic<2 * a_blk + 1>{}, ic<((a + 1) & 1)>{});
                    else frag_one(ic<nxt>{}, ic<FM + b_lo + r - 1>{}, ic<(ks ^ 1)>{});
                }
            });
            CF_SCHED_FENCE();
            {
                // Inline assembly pins the accumulators to the AGPR file: with the builtin the register
                // allocator keeps part of the 64 four-register accumulators of a 128x128 wave tile in
                // VGPRs and copies them to and fro around every MFMA.  An accumulator is touched once
                // per K-step, so two MFMAs on the same registers are never back to back.
                constexpr int h = q / FN, j = q % FN, i = 2 * a + h;
                constexpr int dsel = load_in_gap(q, e_hi - e_lo, NQ);       // the wave-load that goes with this MFMA
                if constexpr (dsel >= 0) {
                    constexpr int e = dsel + e_lo;
                    mma_dma_one(acc[i][j], fb[ks][j], fa[a & 1][h], ic<(e & 1) ? d1 : d0>{}, ic<(e >> 1)>{}, ic<(e & 1)>{});
                } else {
                    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(fb[ks][j]), "v"(fa[a & 1][h]));
                }
            }
            CF_SCHED_FENCE();
        });
    };
    // loads of the pair at (seg, k0) outside the MFMA stream (prologue): all of them, or group 0 only
    auto issue_pair = [&](auto D0, auto D1, auto FIRST_GROUP) __attribute__((always_inline)) {
        prepare_pair();
        static_for<(decltype(FIRST_GROUP)::value ? (NU / NG) * 2 : 2 * NU)>([&](auto E) __attribute__((always_inline)) {
            constexpr int e = decltype(E)::value;
            dma_one(ic<(e & 1) ? decltype(D1)::value : decltype(D0)::value>{}, ic<(e >> 1)>{}, ic<(e & 1)>{});
        });
    };
    // One pair of K-steps s, s+1 in stages ST, ST+1 of the ring of four; the next pair lies in the
    // other two stages, and the loads of the pair after that go back into ST, ST+1 once the barrier
    // has retired them.  The loop body is two pairs, so every stage is a compile-time constant.
    // The loads of a pair are issued in NG groups, the first right after the barrier that frees their
    // stages, which keeps the burst that the load path sees short; the last group still has more
    // than half a pair to land before the next barrier.
    auto pair_body = [&](auto ST) __attribute__((always_inline)) {
        static_for<2 * TM>([&](auto T) __attribute__((always_inline)) {
            constexpr int t = decltype(T)::value;
            if constexpr (t == 2 * TM - 1) {
                prepare_pair();
                wait_vmcnt<0>();        // K-steps s+2, s+3 have landed (nothing else is in flight)
                lds_barrier();          // ... and every wave is done with stages ST and ST+1
            }
            substep(ST, T);
            if constexpr (t == NG - 2) advance_pair();      // the last group of the pair has been issued
        });
    };

    // pairs of K-steps, a segment with an odd number of K-steps padded with a zero K-step
    const int npairs = SPLIT ? (kend - kbeg + 2 * KB - 1) / (2 * KB)
                             : (K0x + 2 * KB - 1) / (2 * KB) + (g.K[1] + 2 * KB - 1) / (2 * KB) +
                                   (g.K[2] + 2 * KB - 1) / (2 * KB);
    // prologue of tile ld: K-steps 0, 1 and the first group of the loads of K-steps 2, 3
    auto start_tile = [&]() __attribute__((always_inline)) {
        seg = 0;
        k0 = 0;
        open_segment(0);
        if (SPLIT) {                    // the block's K range stands for the segment
            k0 = kbeg;
            Kseg = kend;
        }
        issue_pair(ic<0>{}, ic<1>{}, ic<0>{});
        advance_pair();
        issue_pair(ic<2>{}, ic<3>{}, ic<1>{});      // the loop's first sub-steps issue the other groups
    };
    constexpr bool OVERLAP = !SPLIT && !CF32;       // the epilogue leaves the operand stages alone
    if (npairs > 0) start_tile();
    for (;;) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
        if (npairs > 0) {
            // K-steps 0 and 1 have landed.  Everything is waited for, the previous tile's stores
            // included: loads and stores share the counter and retire out of order with respect
            // to each other, so a partial count would say nothing about the loads.
            wait_vmcnt<0>();
            lds_barrier();
            frag_one(ic<0>{}, ic<0>{}, ic<0>{});
            static_for<FN>([&](auto J) __attribute__((always_inline)) { frag_one(ic<0>{}, ic<FM + decltype(J)::value>{}, ic<0>{}); });
            frag_one(ic<0>{}, ic<1>{}, ic<0>{});
            // two pairs per iteration; an odd count runs one pair of zero K-steps (loads past the last
            // segment return zeros)
            for (int p = 0; p < npairs; p += 2) {
                pair_body(ic<0>{});
                pair_body(ic<2>{});
            }
            wait_vmcnt<0>();
            // The MFMAs are inline assembly (see substep), so the compiler does not know that their
            // results are still on the way when the next vector instruction wants to read them: the
            // wait states between a 4-pass MFMA and a reader of its destination are spent here.
            asm volatile("s_nop 15\n\ts_nop 15");
        }
        const TileRef ep = ld;          // the tile that leaves
        const bool has_next = next_tile(ld);
        if (OVERLAP) {
            lds_barrier();              // every wave has read its last fragments: the stages are free
            if (has_next && npairs > 0) start_tile();
        }
        const int m0 = ep.m0, n0 = ep.n0;

    if (SPLIT) {
        // ---- split-K epilogue: fp32 accumulators straight to the block's part ----------
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int m = m0 + wm * (32 * TM) + i * 16 + l16;
                const int n = n0 + wn * (32 * TN) + j * 16 + 4 * g4;
                if (m < Mx && n < ep.N) {                   // N is a multiple of 8
                    float4 o;
                    o.x = acc[i][j][0]; o.y = acc[i][j][1]; o.z = acc[i][j][2]; o.w = acc[i][j][3];
                    *reinterpret_cast<float4*>(part_out + (int64_t)m * ep.N + n) = o;
                }
            }
        break;
    }
    const float alpha = g.alpha;
    if constexpr (CF32) {
        // ---- fp32 epilogue: the two halves of the tile rows (one per wave row) go through LDS in
        // turn, then out as full rows of 16-byte stores, added to beta*C in fp32
        constexpr int HP = BN * 4 + 16;                     // pitch of a staged row of floats
        static_assert((BM / 2) * HP <= GEMM_SMEM, "fp32 staging");
        float* C = static_cast<float*>(ep.C);
        const float beta = g.beta;
        constexpr int CPR = BN / 4, RPP = 256 / CPR;        // 16-byte chunks per row, rows per pass
        const int c = tid % CPR, r0 = tid / CPR;
        const int n = n0 + c * 4;
#pragma unroll 1
        for (int h = 0; h < 2; ++h) {
            lds_barrier();
            if (wm == h) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j) {
                        const int r = i * 16 + l16;
                        const int cc = wn * (32 * TN) + j * 16 + 4 * g4;
                        float4 o;
                        o.x = acc[i][j][0] * alpha; o.y = acc[i][j][1] * alpha;
                        o.z = acc[i][j][2] * alpha; o.w = acc[i][j][3] * alpha;
                        *reinterpret_cast<float4*>(smem + r * HP + cc * 4) = o;
                    }
            }
            lds_barrier();
            if (n < ep.N) {                                  // N is a multiple of 8
                // eight rows per round: all loads of the old values are in flight before the first add
                constexpr int RB = 8;
                static_assert((BM / 2) % (RPP * RB) == 0, "row batches");
#pragma unroll 1
                for (int rb = r0; rb < BM / 2; rb += RPP * RB) {
                    float4 old[RB], val[RB];
#pragma unroll
                    for (int q = 0; q < RB; ++q) {
                        const int m = m0 + h * (BM / 2) + rb + q * RPP;
                        old[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (beta != 0.f && m < Mx) old[q] = *reinterpret_cast<const float4*>(C + (int64_t)m * ep.N + n);
                    }
#pragma unroll
                    for (int q = 0; q < RB; ++q)
                        val[q] = *reinterpret_cast<const float4*>(smem + (rb + q * RPP) * HP + c * 16);
#pragma unroll
                    for (int q = 0; q < RB; ++q) {
                        const int m = m0 + h * (BM / 2) + rb + q * RPP;
                        if (m < Mx) {
                            val[q].x += beta * old[q].x; val[q].y += beta * old[q].y;
                            val[q].z += beta * old[q].z; val[q].w += beta * old[q].w;
                            *reinterpret_cast<float4*>(C + (int64_t)m * ep.N + n) = val[q];
                        }
                    }
                }
            }
        }
        if (!has_next) break;
        lds_barrier();                  // the staging area overlaps the stages
        if (npairs > 0) start_tile();
        continue;
    }
    // ---- epilogue: 32 rows of the wave tile at a time: acc -> bf16 -> the wave's own 8 KB above the
    // four stages -> global with 16-byte stores, whole rows per group of lanes.  The 16-byte chunks
    // of a staged row are XOR-ed with the row number, which keeps both the column-wise writes (a
    // lane holds 4 adjacent columns of one row) and the row-wise reads spread over the banks.  No
    // block barrier: the area is private to the wave and its LDS operations execute in order.
    // The stores go through a buffer descriptor over the whole output matrix, so there is no
    // branch in the stream: rows past M fall outside its range and lanes whose columns lie past
    // N carry an out-of-range offset.
    {
        // bytes of a staged row: 32*TN columns, padded to a power of two of 16-byte chunks (TN = 3:
        // the lanes of the four pad chunks store nothing)
        constexpr int RBY = 64 * (TN == 3 ? 4 : TN);
        constexpr int CPR = RBY / 16, RPP = 64 / CPR;       // 16-byte chunks per row, rows per pass of the wave
        constexpr int NP = 32 / RPP, NV = CPR / RPP;        // passes per 32 rows; distinct swizzle phases
        unsigned char* stg = smem + GEMM_STAGES * STAGE + wave * 8192;
        const __amdgpu_buffer_rsrc_t rc =
            __builtin_amdgcn_make_buffer_rsrc(ep.C, 0, (int)((int64_t)Mx * ep.N * 2), 0x00020000);
        const float beta = g.beta;
        int ln = lane;                                      // as in open_segment: rebuilt per tile, not carried
        asm volatile("" : "+v"(ln));
        const int c = ln % CPR, rl = ln / CPR;
        const int l16 = ln & 15, g4 = ln >> 4;
        const int n = n0 + wn * (32 * TN) + c * 8;
        const unsigned row_bytes = (unsigned)ep.N * 2u;
        // N is a multiple of 8, so a 16-byte chunk lies inside a row or outside it
        const unsigned voff = (n < ep.N && c < 4 * TN)
                                  ? (unsigned)(m0 + wm * (32 * TM) + rl) * row_bytes + (unsigned)n * 2u : OOB_FAST;
        const unsigned char* rd[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) rd[v] = stg + rl * RBY + ((c ^ ((rl + RPP * v) & (CPR - 1))) << 4);
        // a lane's 4 columns of fragment column j are half of the 16-byte chunk 2*j + g4/2 of its row
        unsigned char* const wr = stg + l16 * RBY + (g4 & 1) * 8;
        const int wsw = l16 & (CPR - 1);                    // staged row 16*h + l16, and CPR divides 16
        const int wch = g4 >> 1;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    uint2 o;
                    o.x = pack_bf16x2(acc[2 * i + h][j][0] * alpha, acc[2 * i + h][j][1] * alpha);
                    o.y = pack_bf16x2(acc[2 * i + h][j][2] * alpha, acc[2 * i + h][j][3] * alpha);
                    *reinterpret_cast<uint2*>(wr + h * 16 * RBY + (((2 * j + wch) ^ wsw) << 4)) = o;
                }
            u32x4_t val[NP];
#pragma unroll
            for (int q = 0; q < NP; ++q)
                val[q] = *reinterpret_cast<const u32x4_t*>(rd[q % NV] + q * RPP * RBY);
            if (beta != 0.f) {
#pragma unroll
                for (int q = 0; q < NP; ++q) {
                    const u32x4_t old = __builtin_amdgcn_raw_buffer_load_b128(
                        rc, voff + (unsigned)(i * 32 + q * RPP) * row_bytes, 0, 0);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __uint_as_float(val[q][e] << 16) + beta * __uint_as_float(old[e] << 16);
                        const float hi = __uint_as_float(val[q][e] & 0xFFFF0000u) +
                                         beta * __uint_as_float(old[e] & 0xFFFF0000u);
                        val[q][e] = pack_bf16x2(lo, hi);
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < NP; ++q)
                __builtin_amdgcn_raw_buffer_store_b128(val[q], rc, voff + (unsigned)(i * 32 + q * RPP) * row_bytes, 0, 0);
        }
    }
    if (!has_next) break;
    }   // tile loop
}

// The work items of a launch: the n_full whole tiles first, then the sub-tiles of the remaining
// tiles.  Block b takes items b, b + gridDim.x, ...: with as many blocks as CUs every block runs
// its share of the whole tiles back to back and then at most a few sub-tiles, and the items of
// one block stay on one XCD (item id mod 8 = block id mod 8).
template <int MODE, bool CF32>
__device__ __forceinline__ void gemm_bf16_block(const GemmArgs& g, unsigned char* smem) {
    int Mx = g.M, K0x = g.K[0], n_full = g.n_full, sub = g.sub, tile_n = g.tile_n;
    if (g.n_dev != nullptr) {
        // the kept-token count is a device value: clamp the kept-token dimension to it and (NT: the
        // output shape depends on it) plan the tiles here, as the host does for sizes it knows
        int n = *g.n_dev;
        n = __builtin_amdgcn_readfirstlane(n < 0 ? 0 : n);
        if (MODE == 0) {
            Mx = n < Mx ? n : Mx;
            plan_launch(Mx, g.N, 0, g.c_f32 != 0, g.ngroups, (int)gridDim.x, n_full, sub, tile_n);
            n_full = __builtin_amdgcn_readfirstlane(n_full);
            sub = __builtin_amdgcn_readfirstlane(sub);
            tile_n = __builtin_amdgcn_readfirstlane(tile_n);
        } else {
            K0x = n < K0x ? n : K0x;
        }
    }
    const int tiles_m = (Mx + 255) / 256, tiles_n = (g.N + 255) / 256;
    const int stride = (int)gridDim.x;
    if constexpr (MODE == 0 && !CF32) {
        if (tile_n == 192) {
            // tiles of 256x192, all of one kind: block b takes tiles b, b + gridDim.x, ...
            const int tiles_n192 = (g.N + 191) / 192, n_items = tiles_m * tiles_n192;
            int w = (int)blockIdx.x;
            auto tile = [&](int w, TileRef& t) __attribute__((always_inline)) {
                int bm, bn;
                tile_coords(xcd_order(w, n_items), tiles_m, tiles_n192, bm, bn);
                t.m0 = __builtin_amdgcn_readfirstlane(bm * 256);
                t.n0 = __builtin_amdgcn_readfirstlane(bn * 192);
                t.N = __builtin_amdgcn_readfirstlane(g.N);
                t.B0 = uniform_ptr(g.B[0]);
                t.C = uniform_ptr(g.C);
            };
            TileRef t;
            tile(w, t);
            gemm_tiles<MODE, 4, 3, false, false>(g, Mx, K0x, t, [&](TileRef& nx) __attribute__((always_inline)) {
                w += stride;
                if (w >= n_items) return false;
                tile(w, nx);
                return true;
            }, smem);
            return;
        }
    }
    const int n_items = n_full + (tiles_m * tiles_n - n_full) * sub;
    // item -> tile; false when a sub-tile lies outside the matrix
    auto decode = [&](int w, TileRef& t) __attribute__((always_inline)) {
        int bm, bn, m0, n0;
        if (w < n_full) {
            tile_coords(xcd_order(w, n_full), tiles_m, tiles_n, bm, bn);
            m0 = bm * 256;
            n0 = bn * 256;
        } else {
            const int cut = sub;
            const int j = xcd_order(w - n_full, n_items - n_full);
            const int part = j % cut;
            tile_coords(n_full + j / cut, tiles_m, tiles_n, bm, bn);
            m0 = bm * 256 + (cut == 4 ? (part >> 1) * 128 : 0);
            n0 = bn * 256 + (cut == 4 ? (part & 1) * 128 : (cut == 2 ? part * 128 : 0));
            if (m0 >= Mx || n0 >= g.N) return false;
        }
        t.B0 = g.B[0];
        t.C = g.C;
        t.N = g.N;
        if (g.ngroups > 1) {
            // the tile's column group: rebase the B operand, the output and the column range on it
            const int j = n0 < g.Ng[0] ? 0 : (n0 < g.Ng[0] + g.Ng[1] ? 1 : 2);
            const int off = j == 0 ? 0 : (j == 1 ? g.Ng[0] : g.Ng[0] + g.Ng[1]);
            t.B0 = j == 0 ? g.Bg[0] : (j == 1 ? g.Bg[1] : g.Bg[2]);
            t.C = j == 0 ? g.Cg[0] : (j == 1 ? g.Cg[1] : g.Cg[2]);
            t.N = j == 0 ? g.Ng[0] : (j == 1 ? g.Ng[1] : g.Ng[2]);
            n0 -= off;
        }
        // every field is the same in all lanes: say so, which keeps the address arithmetic of the
        // tile's prologue on the scalar unit
        t.m0 = __builtin_amdgcn_readfirstlane(m0);
        t.n0 = __builtin_amdgcn_readfirstlane(n0);
        t.N = __builtin_amdgcn_readfirstlane(t.N);
        t.B0 = uniform_ptr(t.B0);
        t.C = uniform_ptr(t.C);
        return true;
    };
    int w = (int)blockIdx.x;
    TileRef t;
    // the next item of this block below `end` that is a tile
    auto advance = [&](int end) __attribute__((always_inline)) {
        for (w += stride; w < end; w += stride)
            if (decode(w, t)) return true;
        return false;
    };
    if (w < n_full) {         // whole tiles
        decode(w, t);
        gemm_tiles<MODE, 4, 4, false, CF32>(g, Mx, K0x, t, [&](TileRef& nx) __attribute__((always_inline)) {
            if (!advance(n_full)) return false;
            nx = t;
            return true;
        }, smem);
    }
    // sub-tiles: w is now this block's first item at or past n_full
    bool have = false;
    for (; w < n_items; w += stride)
        if (decode(w, t)) { have = true; break; }
    if (!have) return;
    auto next_sub = [&](TileRef& nx) __attribute__((always_inline)) {
        if (!advance(n_items)) return false;
        nx = t;
        return true;
    };
    if (sub == 1) gemm_tiles<MODE, 4, 4, false, CF32>(g, Mx, K0x, t, next_sub, smem);
    else if (sub == 2) gemm_tiles<MODE, 4, 2, false, CF32>(g, Mx, K0x, t, next_sub, smem);
    else gemm_tiles<MODE, 2, 2, false, CF32>(g, Mx, K0x, t, next_sub, smem);
}

template <int MODE>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs g) {
    extern __shared__ __align__(16) unsigned char smem[];
    gemm_bf16_block<MODE, false>(g, smem);
}

// The same with fp32 output (main-gradient buffers): C is float, added to beta*C without rounding.
template <int MODE>
__global__ __launch_bounds__(256) void gemm_bf16_f32out_kernel(GemmArgs g) {
    extern __shared__ __align__(16) unsigned char smem[];
    gemm_bf16_block<MODE, true>(g, smem);
}

// Split-K variant for outputs with too few tiles to fill the chip (a skinny M or N with a long
// K: the products with a rank-r adapter matrix).  grid = (128x128 tiles, parts); part p contracts
// k in [p*kchunk, (p+1)*kchunk) into partial[p]; splitk_reduce_kernel sums the parts in a fixed
// order, so the result does not depend on scheduling.
template <int MODE>
__global__ __launch_bounds__(256) void gemm_bf16_splitk_kernel(GemmArgs g, float* partial, int kchunk) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tiles_m = (g.M + 127) / 128;
    const int m0 = ((int)blockIdx.x % tiles_m) * 128, n0 = ((int)blockIdx.x / tiles_m) * 128;
    // a device-side kept-token count bounds M (mode NT) or K (mode TN); the launch was planned for the
    // host's upper bound, so a block may find its rows or its K range empty: it then stores nothing
    // (NT; the reduction skips those rows too) or a tile of zeros (TN)
    int Mx = g.M, Kx = g.K[0];
    if (g.n_dev != nullptr) {
        const int n = max(*g.n_dev, 0);
        if (MODE == 0) Mx = min(Mx, n);
        else Kx = min(Kx, n);
    }
    const int kbeg = (int)blockIdx.y * kchunk;
    const int kend = max(kbeg, min(Kx, kbeg + kchunk));
    if (MODE == 0 && m0 >= Mx) return;
    const TileRef t{m0, n0, g.N, g.B[0], g.C};
    gemm_tiles<MODE, 2, 2, true, false>(g, Mx, Kx, t, [](TileRef&) { return false; }, smem, kbeg, kend,
                                        partial + (int64_t)blockIdx.y * g.M * g.N);
}

// C[m, n..n+7] = alpha * sum_p partial[p][m, n..n+7] + beta * C
// rows_dev (nullable): the live number of rows of C on the device (mode NT with a device-side count);
// rows past it have no partials and are left alone.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, bf16_t* __restrict__ C,
                                                            int64_t mn, int parts, float alpha, float beta,
                                                            const int32_t* __restrict__ rows_dev, int ncols) {
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (e >= mn) return;
    if (rows_dev != nullptr && e >= (int64_t)max(*rows_dev, 0) * ncols) return;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int p = 0; p < parts; ++p) {
        const float4 a = *reinterpret_cast<const float4*>(partial + p * mn + e);
        const float4 b = *reinterpret_cast<const float4*>(partial + p * mn + e + 4);
        s[0] += a.x; s[1] += a.y; s[2] += a.z; s[3] += a.w;
        s[4] += b.x; s[5] += b.y; s[6] += b.z; s[7] += b.w;
    }
    u32x4_t val;
    if (beta != 0.f) {
        const u32x4_t old = *reinterpret_cast<const u32x4_t*>(C + e);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            val[q] = pack_bf16x2(alpha * s[2 * q] + beta * __uint_as_float(old[q] << 16),
                                 alpha * s[2 * q + 1] + beta * __uint_as_float(old[q] & 0xFFFF0000u));
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) val[q] = pack_bf16x2(alpha * s[2 * q], alpha * s[2 * q + 1]);
    }
    *reinterpret_cast<u32x4_t*>(C + e) = val;
}

// ---------------------------------------------------------------------------
// fp32 check-mode GEMM: 64x64 tile, 16-wide K step, 4x4 outputs per thread
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g) {
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64 + 4];
    const int tid = threadIdx.x;
    const int tiles_m = (g.M + 63) / 64;        // of the upper bound: the grid was sized for it
    const int m0 = (blockIdx.x % tiles_m) * 64, n0 = (blockIdx.x / tiles_m) * 64;
    if (g.n_dev != nullptr) {
        const int n = live_rows(MODE == 0 ? g.M : g.K[0], g.n_dev);
        if (MODE == 0) g.M = n;
        else g.K[0] = n;
        if (m0 >= g.M) return;
    }
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
                if (ka && m0 + r < g.M) {
                    const int64_t arow = (MODE == 0 && s == 0 && g.a_idx != nullptr) ? g.a_idx[m0 + r] : m0 + r;
                    av = MODE == 0 ? A[arow * K + k0 + kk] : A[(int64_t)(k0 + kk) * g.M + m0 + r];
                }
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
            *p = (g.beta != 0.f) ? g.alpha * acc[i][j] + g.beta * *p : g.alpha * acc[i][j];
        }
    }
}


// Number of K parts for a split-K launch (0: use the ordinary kernel) and the K range of a part.
// Splitting pays when the 128x128 tiles cover at most half of the CUs and K is long enough that
// every part still runs several K-steps.
static int plan_splitk(const GemmArgs& g, int n_cu, size_t ws_bytes, int& kchunk) {
    if (g.nseg != 1 || g.ngroups > 1 || g.c_f32) return 0;
    const int K = g.K[0];
    const int tiles = ceil_div(g.M, 128) * ceil_div(g.N, 128);
    if (tiles * 2 > n_cu || K < 1024) return 0;
    const size_t per_part = (size_t)g.M * g.N * sizeof(float);
    int parts = std::min(std::min(n_cu / tiles, K / 256), 32);
    parts = (int)std::min<size_t>((size_t)parts, ws_bytes / per_part);
    if (parts < 2) return 0;
    kchunk = ceil_div(ceil_div(K, parts), 64) * 64;
    return ceil_div(K, kchunk);
}

template <int MODE>
static hipError_t launch_bf16_splitk(GemmArgs& g, int parts, int kchunk, float* partial, hipStream_t st) {
    static std::atomic<uint64_t> lds_ok{0};
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_bf16_splitk_kernel<MODE>), GEMM_SMEM, lds_ok);
    if (e != hipSuccess) return e;
    const dim3 grid(ceil_div(g.M, 128) * ceil_div(g.N, 128), parts);
    gemm_bf16_splitk_kernel<MODE><<<grid, 256, GEMM_SMEM, st>>>(g, partial, kchunk);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t mn = (int64_t)g.M * g.N;
    splitk_reduce_kernel<<<(unsigned)ceil_div(mn / 8, (int64_t)256), 256, 0, st>>>(
        partial, static_cast<bf16_t*>(g.C), mn, parts, g.alpha, g.beta, MODE == 0 ? g.n_dev : nullptr, g.N);
    return hipGetLastError();
}

template <int MODE>
static hipError_t launch_bf16(GemmArgs& g, hipStream_t st) {
    static std::atomic<uint64_t> lds_ok{0}, lds_ok_f32{0};
    hipError_t e = g.c_f32 ? allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_bf16_f32out_kernel<MODE>), GEMM_SMEM, lds_ok_f32)
                           : allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_bf16_kernel<MODE>), GEMM_SMEM, lds_ok);
    if (e != hipSuccess) return e;
    const int items = plan_launch(g.M, g.N, MODE, g.c_f32 != 0, g.ngroups, compute_units(), g.n_full, g.sub, g.tile_n);
    // a block walks through its items; with a device-side count the blocks plan for themselves (for
    // as many blocks as CUs) and those without an item leave at once
    const int grid = g.n_dev != nullptr ? compute_units() : std::min(items, compute_units());
    if (g.c_f32) gemm_bf16_f32out_kernel<MODE><<<grid, 256, GEMM_SMEM, st>>>(g);
    else gemm_bf16_kernel<MODE><<<grid, 256, GEMM_SMEM, st>>>(g);
    return hipGetLastError();
}

hipError_t launch_gemm(int dtype, int mode, const GemmSeg* segs, int nseg, void* C, int M, int N,
                       float beta, hipStream_t st, float alpha, void* splitk_ws, size_t splitk_bytes,
                       bool c_f32, const int32_t* n_dev, const int32_t* a_idx, int64_t a_rows) {
    if (M <= 0 || N <= 0) return hipSuccess;
    if (a_idx != nullptr && (mode != 0 || a_rows <= 0)) return hipErrorInvalidValue;
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
    g.C = C; g.M = M; g.N = N; g.beta = beta; g.alpha = alpha; g.n_full = 0; g.sub = 1; g.tile_n = 256;
    g.c_f32 = (c_f32 && dtype == CF_BF16) ? 1 : 0;
    g.ngroups = 1;
    for (int j = 0; j < 3; ++j) { g.Bg[j] = nullptr; g.Cg[j] = nullptr; g.Ng[j] = 0; }
    g.n_dev = n_dev; g.a_idx = a_idx; g.a_rows = a_rows;
    // with a device-side count the kept-token dimension must be that of segment 0 (mode TN) and no
    // segment may have been dropped
    if (n_dev != nullptr && (g.nseg != nseg || (mode == 1 && nseg != 1))) return hipErrorInvalidValue;
    if (g.nseg == 0) {
        // empty contraction: C = beta*C; only beta in {0,1} is supported by the API
        if (beta == 0.f) return launch_fill_zero(C, (size_t)M * N * (c_f32 ? 4 : dtype_size(dtype)), st);
        return hipSuccess;
    }
    if (dtype == CF_BF16) {
        // per-lane load and store offsets are 32-bit with the upper half reserved for "out of range"
        for (int s = 0; s < g.nseg; ++s)
            if ((int64_t)M * g.K[s] * 2 >= ((int64_t)1 << 31) || (int64_t)N * g.K[s] * 2 >= ((int64_t)1 << 31))
                return hipErrorInvalidValue;
        if (a_idx != nullptr && a_rows * g.K[0] * 2 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
        if (((int64_t)M + 256) * N * 2 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    }
    if (dtype == CF_F32) {
        const int grid = ceil_div(M, 64) * ceil_div(N, 64);
        if (mode == 0) gemm_f32_kernel<0><<<grid, 256, 0, st>>>(g);
        else gemm_f32_kernel<1><<<grid, 256, 0, st>>>(g);
        return hipGetLastError();
    }
    if (splitk_ws != nullptr && a_idx == nullptr) {
        int kchunk = 0;
        const int parts = plan_splitk(g, compute_units(), splitk_bytes, kchunk);
        if (parts >= 2)
            return mode == 0 ? launch_bf16_splitk<0>(g, parts, kchunk, static_cast<float*>(splitk_ws), st)
                             : launch_bf16_splitk<1>(g, parts, kchunk, static_cast<float*>(splitk_ws), st);
    }
    return mode == 0 ? launch_bf16<0>(g, st) : launch_bf16<1>(g, st);
}

bool gemm_tn_groups_supported(int dtype, int K, int ngroups, const int* Ng) {
    if (dtype != CF_BF16 || K <= 0 || ngroups < 2 || ngroups > 3) return false;
    for (int j = 0; j < ngroups; ++j)
        if (Ng[j] <= 0 || Ng[j] % 256 != 0) return false;
    return true;
}

hipError_t launch_gemm_tn_groups(const void* A, int K, int M, int ngroups, const void* const* Bg,
                                 void* const* Cg, const int* Ng, hipStream_t st, float beta, bool c_f32,
                                 const int32_t* n_dev) {
    if (M <= 0) return hipSuccess;
    GemmArgs g;
    int N = 0;
    for (int j = 0; j < 3; ++j) {
        g.Bg[j] = j < ngroups ? Bg[j] : nullptr;
        g.Cg[j] = j < ngroups ? Cg[j] : nullptr;
        g.Ng[j] = j < ngroups ? Ng[j] : 0;
        N += g.Ng[j];
        if ((int64_t)g.Ng[j] * K * 2 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    }
    if ((int64_t)M * K * 2 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    for (int j = 0; j < ngroups; ++j)
        if (((int64_t)M + 256) * Ng[j] * 2 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    g.ngroups = ngroups;
    g.A[0] = A; g.B[0] = Bg[0]; g.K[0] = K; g.nseg = 1;
    for (int s = 1; s < 3; ++s) { g.A[s] = nullptr; g.B[s] = nullptr; g.K[s] = 0; }
    g.C = Cg[0]; g.M = M; g.N = N; g.beta = beta; g.alpha = 1.f; g.n_full = 0; g.sub = 1; g.tile_n = 256;
    g.c_f32 = c_f32 ? 1 : 0;
    g.n_dev = n_dev; g.a_idx = nullptr; g.a_rows = 0;
    return launch_bf16<1>(g, st);
}

}  // namespace cf
