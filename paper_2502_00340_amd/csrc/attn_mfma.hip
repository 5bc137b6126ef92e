// Filtered attention backward on the matrix cores (Sec. 3.1, Eq. 3-4), bf16 in,
// fp32 softmax statistics and accumulators.  Two deterministic kernels, no atomics:
//
//   dQ kernel   (Eq. 3 dS*K-hat + Eq. 4 dS*K-check in one pass): a block owns 128
//               kept queries of one (sequence, query head) and walks over ALL key
//               tiles up to the last query's original position; P is rebuilt
//               from the saved LSE, so filtered keys contribute exactly as in
//               the forward pass.
//   dK/dV kernel (Eq. 3): a block owns 128 KEPT keys of one (sequence, QUERY head) and
//               walks over the kept queries at or after them; rows of filtered
//               tokens are never formed.  Kept rows are in position order, so
//               causality is "compact query index >= compact key index".  With
//               grouped heads each query head writes an fp32 partial and a small
//               kernel sums the G partials of a KV head in a fixed order.
//
// Block order: the (head, sequence) index varies fastest and the tile index
// slowest with the heaviest tiles first, so that the 8 XCDs (block id mod 8)
// receive equal shares of every tile weight and the tail of the launch is made
// of light blocks.  K/V (dQ kernel) and Q/dO (dK/dV kernel) tiles go from global
// memory straight into LDS (16 bytes per lane), one tile ahead of the MFMAs.
//
// Operand orientation is chosen so that no score tile ever goes through LDS:
// the dQ kernel forms S^T = K*Q^T (accumulator lane = query, registers = keys),
// which is already the A-operand layout of dQ += dS*K; the dK/dV kernel forms
// S = Q*K^T (lane = key, registers = queries), the A-operand layout of
// dV += P^T*dO and dK += dS^T*Q.  The second operand of those products has the
// token dimension as K; it is fetched from the same [token][d] LDS tile with
// the LDS transpose read (ds_read_b64_tr_b16).
//
// 32x32x16 bf16 MFMA operand layout (lane l, slot = l%32, hh = l/32):
//   A: row = slot,  k = 8*hh + e (e = 0..7)      B: col = slot, k = 8*hh + e
//   D: col = slot,  row = 8*(v/4) + 4*hh + v%4   (v = 0..15)
// so accumulator registers 8j..8j+7 of a lane, used as one A/B fragment, carry
// rows {16j + 4hh + e, 16j + 8 + 4hh + e}; the transpose reads fetch exactly
// those rows for the other operand.
#include "common.h"
#include "mfma_util.h"

namespace cf {

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;

static constexpr float LOG2E = 1.4426950408889634f;

struct AttnParams {
    const bf16_t *q_kept, *k_full, *v_full, *do_kept;
    const float* stat;             // [2][Hq][n_kept]: log2(e)*LSE and D = rowsum(dO*O) of every kept row and head
    const int32_t *idx, *cu_kept;
    bf16_t *dq_kept, *dk_kept, *dv_kept;
    float *dk_part, *dv_part;      // [G/hp][n_kept][Hkv*d] fp32 partials, one per block of hp query heads (G > hp only)
    int n_cu;                      // compute units of the device (the dK/dV kernel sizes its blocks' work by it)
    int B, S, Hq, Hkv;
    int n_kept;                    // rows that the compact buffers are laid out for (the stride of stat and of the partials)
    const int32_t* n_dev;          // nullable: the live row count on the device, at most n_kept
    float scale;
};

// Query heads of one KV group that a dK/dV block walks through: the largest divisor of the group size G
// that still leaves about two blocks per CU (a block costs between one and `tiles` steps and blocks are
// handed out heaviest first, so two per CU already balance); every head more in a block saves that
// block's fixed cost once and one fp32 partial.  A function of the LIVE row count, which only the
// device may know: the dK/dV blocks and the reduction evaluate it themselves and agree.
__host__ __device__ inline int attn_heads_per_block(int n_rows, int Hq, int G, int n_cu) {
    const int64_t tile_rows = (n_rows + 127) / 128;             // key tiles over all sequences, roughly
    for (int c = G; c > 1; --c)
        if (G % c == 0 && tile_rows * (Hq / c) >= 2 * (int64_t)n_cu) return c;
    return 1;
}

// Compact rows [begin, end) of sequence b.  The prefix counts are clamped to the live row count, so a
// mask that keeps more tokens than the buffers were sized for cannot send a block past their end.
__device__ __forceinline__ void seq_range(const AttnParams& p, int b, int& begin, int& end) {
    if (p.cu_kept == nullptr) {
        begin = b * p.S;
        end = (b + 1) * p.S;
        return;
    }
    const int n = live_rows(p.n_kept, p.n_dev);
    begin = min(p.cu_kept[b], n);
    end = min(p.cu_kept[b + 1], n);
}

// 16-byte chunk swizzle of a [rows][D] bf16 tile: makes both the row-fragment
// reads (16 consecutive rows, same chunk) and the transpose reads (4 rows x 4
// consecutive chunks per half wave) bank-conflict free.
template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk) {
    const int g = (D == 128) ? (((row & 3) << 2) | ((row >> 2) & 3))
                             : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
    return row * (D * 2) + ((chunk ^ g) << 4);
}

__device__ __forceinline__ unsigned pack2(float lo, float hi) {
    bf16x2_t v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(unsigned, v);
}

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& a, int j) {
    uint4 u;
    u.x = pack2(a[8 * j + 0], a[8 * j + 1]);
    u.y = pack2(a[8 * j + 2], a[8 * j + 3]);
    u.z = pack2(a[8 * j + 4], a[8 * j + 5]);
    u.w = pack2(a[8 * j + 6], a[8 * j + 7]);
    return __builtin_bit_cast(bf16x8_t, u);
}

// A/B fragment with the tile row as the MFMA row/col and d as K
template <int D>
__device__ __forceinline__ bf16x8_t frag_rows(const unsigned char* tile, int row, int ks, int hh) {
    return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(tile + tile_off<D>(row, ks * 2 + hh)));
}

// B fragment with d as the MFMA column and the tile row (token) as K:
// rows row0 + 4hh + {0..3} and row0 + 8 + 4hh + {0..3}, columns nt*32 + slot
template <int D>
__device__ __forceinline__ bf16x8_t frag_tokens(const unsigned char* tile, int row0, int nt, int lane) {
    const int hh = lane >> 5;
    const int r = row0 + 4 * hh + ((lane & 15) >> 2);
    const int chunk = nt * 4 + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    const int sub = (lane & 1) * 8;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4_ptr)(tile + tile_off<D>(r, chunk) + sub));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4_ptr)(tile + tile_off<D>(r + 8, chunk) + sub));
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;
    s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, both);
}

// global -> LDS: a [64][D] tile goes in as 1 KB wave-loads (16 bytes per lane): wave w, load i fills
// LDS bytes [(4*i + w) KB, +1 KB) of the tile, i.e. 1024/(2D) rows, and a lane fetches the global chunk
// that belongs in its (swizzled) LDS slot.  Rows outside the source's descriptor range arrive as zeros.

// ---------------------------------------------------------------------------
// dQ kernel
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 2) void attn_dq_kernel(AttnParams p) {
    constexpr int KS = D / 16, NT = D / 32;
    constexpr int TILE = 64 * D * 2;            // one 64-token tile in bytes
    constexpr int NLD = D / 32;                 // wave-loads per wave per tile
    extern __shared__ __align__(16) unsigned char smem[];   // [2 stages][K tile, V tile]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slot = lane & 31, hh = lane >> 5;
    const int h = blockIdx.x % p.Hq, b = blockIdx.x / p.Hq, g = h / (p.Hq / p.Hkv);
    const int Nq = p.Hq * D, Nkv = p.Hkv * D;
    int seq_begin, seq_end;
    seq_range(p, b, seq_begin, seq_end);
    const int cnt = seq_end - seq_begin;
    // heaviest (latest) query tiles of the sequence first; the grid is sized for an upper bound of the
    // row count, and the blocks past this sequence's tiles come last in the launch order
    const int seq_tiles = (cnt + 127) / 128;
    if ((int)blockIdx.y >= seq_tiles) return;
    const int qt = seq_tiles - 1 - blockIdx.y;
    const int j0 = seq_begin + qt * 128;
    const int rows_in_tile = min(128, cnt - qt * 128);

    // this lane's query
    const int jq = j0 + wave * 32 + slot;
    const bool qvalid = wave * 32 + slot < rows_in_tile;
    const int pos = qvalid ? (p.idx ? p.idx[jq] : jq) - b * p.S : -1;
    const float lse2 = qvalid ? p.stat[(int64_t)h * p.n_kept + jq] : 0.f;
    const float Dq = qvalid ? p.stat[(int64_t)(p.Hq + h) * p.n_kept + jq] : 0.f;
    bf16x8_t qf[KS], dof[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        uint4 a = make_uint4(0, 0, 0, 0), c = make_uint4(0, 0, 0, 0);
        if (qvalid) {
            a = *reinterpret_cast<const uint4*>(p.q_kept + (int64_t)jq * Nq + h * D + ks * 16 + hh * 8);
            c = *reinterpret_cast<const uint4*>(p.do_kept + (int64_t)jq * Nq + h * D + ks * 16 + hh * 8);
        }
        qf[ks] = __builtin_bit_cast(bf16x8_t, a);
        dof[ks] = __builtin_bit_cast(bf16x8_t, c);
    }
    const int jlast = j0 + rows_in_tile - 1;
    const int maxpos = (p.idx ? p.idx[jlast] : jlast) - b * p.S;
    const int nkt = maxpos / 64 + 1;
    // positions of the wave's last and first query: key tiles past the former are skipped, key tiles
    // that end at or before the latter are visible to every query of the wave and need no mask
    int wave_maxpos = -1, wave_minpos = -1;
    {
        const int wrows = min(32, rows_in_tile - wave * 32);
        if (wrows > 0) {
            const int jw = j0 + wave * 32 + wrows - 1;
            wave_maxpos = (p.idx ? p.idx[jw] : jw) - b * p.S;
            wave_minpos = (p.idx ? p.idx[j0 + wave * 32] : j0 + wave * 32) - b * p.S;
        }
    }
    const float scale2 = p.scale * LOG2E;

    f32x16_t acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nt][v] = 0.f;

    // K and V of this sequence and KV head: rows are Nkv*2 bytes apart.  A tile is loaded whole: rows past
    // the last query's position are later keys of the same sequence (masked out below) or lie outside
    // the descriptor's range (zeros).
    const i32x4_t rsK = make_rsrc(p.k_full + ((int64_t)b * p.S) * Nkv + g * D, ((int64_t)p.S * Nkv - g * D) * 2);
    const i32x4_t rsV = make_rsrc(p.v_full + ((int64_t)b * p.S) * Nkv + g * D, ((int64_t)p.S * Nkv - g * D) * 2);
    const unsigned lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(smem));
    // per-lane offset of a tile's first load inside a 64-row tile (row * stride + swizzled chunk): it never
    // changes, and load i lies 4*i*RPL rows further on with the same swizzle term
    constexpr int NCH = D / 8, RPL = 64 / NCH;
    unsigned voff0;
    {
        const int row = wave * RPL + lane / NCH;
        const int pc = lane % NCH;
        const int sw = (D == 128) ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
        voff0 = (unsigned)row * (unsigned)(Nkv * 2) + (unsigned)((pc ^ sw) << 4);
    }
    const unsigned wave_lds = __builtin_amdgcn_readfirstlane(lds0 + (unsigned)wave * 1024u);   // scalar: the wave's 1 KB slot
    auto issue_kv = [&](int kt, int stage) __attribute__((always_inline)) {
        const unsigned sk = wave_lds + stage * 2 * TILE;
        const unsigned step = (unsigned)(4 * RPL) * (unsigned)(Nkv * 2);
        const unsigned base = (unsigned)(kt * 64) * (unsigned)(Nkv * 2);
#pragma unroll
        for (int i = 0; i < NLD; ++i) dma16(sk + 4 * i * 1024, rsK, voff0 + (base + i * step));
#pragma unroll
        for (int i = 0; i < NLD; ++i) dma16(sk + TILE + 4 * i * 1024, rsV, voff0 + (base + i * step));
    };
    // One 64-key tile in the LDS stage at sk.  MASKED: some key of the tile lies after some query of the
    // wave; the other tiles (most of them) spend no instruction on the mask.
    // One 32-key half of the tile at a time keeps the score registers at 2 x 16.  The LDS fragments of an
    // MFMA are read while the previous MFMAs run (one step ahead).  (Fragment addresses are rebuilt per
    // read: with two waves per SIMD the register file has no room to keep them at d = 128.)
    auto tile = [&](auto MASKED_, const int kt, const unsigned char* sk) __attribute__((always_inline)) {
        constexpr bool masked = decltype(MASKED_)::value != 0;
        const unsigned char* sv = sk + TILE;
        bf16x8_t fa[2][2], fc[2];
        auto load_a = [&](int mt, int ks, int buf) __attribute__((always_inline)) {
            fa[buf][0] = frag_rows<D>(sk, mt * 32 + slot, ks, hh);
            fa[buf][1] = frag_rows<D>(sv, mt * 32 + slot, ks, hh);
        };
        auto load_c = [&](int mt, int c, int buf) __attribute__((always_inline)) {
            fc[buf] = frag_tokens<D>(sk, mt * 32 + 16 * (c / NT), c % NT, lane);
        };
        load_a(0, 0, 0);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f32x16_t st, dpt;
#pragma unroll
            for (int v = 0; v < 16; ++v) { st[v] = 0.f; dpt[v] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks + 1 < KS) load_a(mt, ks + 1, (ks + 1) & 1);
                else load_c(mt, 0, 0);
                CF_SCHED_FENCE();
                st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][0], qf[ks], st, 0, 0, 0);
                dpt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][1], dof[ks], dpt, 0, 0, 0);
                CF_SCHED_FENCE();
            }
            // dS^T = P^T o (dP^T - D): lane = query, register = key
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float pr = __builtin_amdgcn_exp2f(st[v] * scale2 - lse2);
                if (masked) {
                    const int key = kt * 64 + mt * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
                    pr = key <= pos ? pr : 0.f;
                }
                st[v] = pr * (dpt[v] - Dq);
            }
            const bf16x8_t a0 = pack8(st, 0), a1 = pack8(st, 1);
#pragma unroll
            for (int c = 0; c < 2 * NT; ++c) {
                if (c + 1 < 2 * NT) load_c(mt, c + 1, (c + 1) & 1);
                else if (mt == 0) load_a(1, 0, 0);
                CF_SCHED_FENCE();
                acc[c % NT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(c < NT ? a0 : a1, fc[c & 1], acc[c % NT], 0, 0, 0);
                CF_SCHED_FENCE();
            }
        }
    };

    issue_kv(0, 0);
    wait_vmcnt<0>();
    lds_barrier();
    for (int kt = 0; kt < nkt; ++kt) {
        if (kt + 1 < nkt) issue_kv(kt + 1, (kt + 1) & 1);
        if (kt * 64 <= wave_maxpos) {
            // a query that does not exist (a ragged last wave) has position -1 and is masked in every tile
            const bool clear = kt * 64 + 63 <= wave_minpos && wave * 32 + 32 <= rows_in_tile;
            const unsigned char* sk = smem + (kt & 1) * 2 * TILE;
            if (clear) tile(ic<0>{}, kt, sk);
            else tile(ic<1>{}, kt, sk);
        }
        wait_vmcnt<0>();
        lds_barrier();
    }

    // dq[query][d]: lane = d column, registers = query rows
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = wave * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
            if (r < rows_in_tile)
                p.dq_kept[(int64_t)(j0 + r) * Nq + h * D + nt * 32 + slot] = f32_to_bf16(acc[nt][v] * p.scale);
        }
    }
}

// ---------------------------------------------------------------------------
// dK/dV kernel: one (key tile, query head) per block
// ---------------------------------------------------------------------------
// Slot order of an iteration of the kernel's pipeline (2*KS positions, KS "A" slots and KS "C" slots;
// see the kernel): odd iterations alternate A, C; even iterations put all C slots into the first
// 3*KS/2 positions, every third of which is an A slot, and the remaining A slots behind them.
__host__ __device__ constexpr bool dkv_is_a(int KS, bool even, int p) {
    return even ? (p < 3 * KS / 2 ? (p % 3 == 1) : true) : (p % 2 == 0);
}
__host__ __device__ constexpr int dkv_slot_index(int KS, bool even, int p) {
    int n = 0;
    for (int q = 0; q < p; ++q) n += (dkv_is_a(KS, even, q) == dkv_is_a(KS, even, p)) ? 1 : 0;
    return n;
}

template <int D>
__global__ __launch_bounds__(256, 1) void attn_dkv_kernel(AttnParams p) {
    constexpr int KS = D / 16, NT = D / 32;
    constexpr int TILE = 64 * D * 2;
    constexpr int STAGE = 2 * TILE + 512;       // Q tile, dO tile, lse2[64], D[64]
    extern __shared__ __align__(16) unsigned char smem[];

    // the wave number is the same in all lanes: saying so keeps everything derived from it in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slot = lane & 31, hh = lane >> 5;
    const int G = p.Hq / p.Hkv;
    const int HP = attn_heads_per_block(live_rows(p.n_kept, p.n_dev), p.Hq, G, p.n_cu);
    // The grid is one-dimensional and has a block per (key tile, sequence, query head).  Only nhb * B blocks
    // per key tile are needed; they are numbered first, key tile by key tile (heaviest first), so the blocks
    // without work all come at the end of the launch order instead of between the working ones (a block
    // needs a whole CU's LDS even to find out that it has nothing to do).
    const int nhb = p.Hq / HP;                      // head blocks per sequence
    const int per_tile = nhb * p.B;
    const int kt = blockIdx.x / per_tile, bx = blockIdx.x % per_tile;
    if (kt >= (int)gridDim.x / (p.Hq * p.B)) return;
    const int h0 = (bx % nhb) * HP, b = bx / nhb, g = h0 / G;
    const int Nq = p.Hq * D, Nkv = p.Hkv * D;
    int seq_begin, seq_end;
    seq_range(p, b, seq_begin, seq_end);
    const int cnt = seq_end - seq_begin;
    if (kt * 128 >= cnt) return;                    // early key tiles see the most queries: heaviest first
    const int c0 = seq_begin + kt * 128;            // compact row of the tile's first key
    const int keys_in_tile = min(128, cnt - kt * 128);

    // this lane's key
    const int jk = c0 + wave * 32 + slot;
    const bool kvalid = wave * 32 + slot < keys_in_tile;
    bf16x8_t kf[KS], vf[KS];
    {
        const int64_t tok = kvalid ? (p.idx ? p.idx[jk] : jk) : 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint4 a = make_uint4(0, 0, 0, 0), c = make_uint4(0, 0, 0, 0);
            if (kvalid) {
                a = *reinterpret_cast<const uint4*>(p.k_full + tok * Nkv + g * D + ks * 16 + hh * 8);
                c = *reinterpret_cast<const uint4*>(p.v_full + tok * Nkv + g * D + ks * 16 + hh * 8);
            }
            kf[ks] = __builtin_bit_cast(bf16x8_t, a);
            vf[ks] = __builtin_bit_cast(bf16x8_t, c);
        }
    }
    const float scale2 = p.scale * LOG2E;
    const int steps = (seq_end - c0 + 63) / 64;     // query tiles from the first key to the sequence end

    f32x16_t dk[NT], dv[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) { dk[nt][v] = 0.f; dv[nt][v] = 0.f; }

    // Q and dO rows of this sequence from its first key on, the current head's columns (set per head below)
    i32x4_t rsQ, rsO, rsL, rsD;
    auto open_head = [&](int h) __attribute__((always_inline)) {
        rsQ = make_rsrc(p.q_kept + (int64_t)c0 * Nq + h * D, ((int64_t)(seq_end - c0) * Nq - h * D) * 2);
        rsO = make_rsrc(p.do_kept + (int64_t)c0 * Nq + h * D, ((int64_t)(seq_end - c0) * Nq - h * D) * 2);
        rsL = make_rsrc(p.stat + (int64_t)h * p.n_kept + c0, (int64_t)(seq_end - c0) * 4);
        rsD = make_rsrc(p.stat + (int64_t)(p.Hq + h) * p.n_kept + c0, (int64_t)(seq_end - c0) * 4);
    };
    const unsigned lds0 = __builtin_amdgcn_readfirstlane(lds_addr_of(smem));
    // Per-lane byte offsets of the fragment reads inside a 64-row tile, fixed for the whole kernel:
    // row fragments (this lane's row of a 32-row half, d chunk ks) and token fragments (d block nt,
    // low / high four rows of a 16-row block).  The XOR swizzle is folded in here, so a read in the
    // loop is "stage base + this + compile-time offset".
    unsigned ra[KS], ta[NT][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ra[ks] = (unsigned)tile_off<D>(slot, ks * 2 + hh);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int r = 4 * hh + ((lane & 15) >> 2);
        const int chunk = nt * 4 + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
        ta[nt][0] = (unsigned)tile_off<D>(r, chunk) + (lane & 1) * 8;
        ta[nt][1] = (unsigned)tile_off<D>(r + 8, chunk) + (lane & 1) * 8;
    }
    // ---- global -> LDS.  Per-lane offsets of a tile's loads inside a 64-row step (row * stride +
    // swizzled chunk) never change; the step's row offset is added per step.  Rows past the sequence
    // end lie outside the descriptors' ranges and arrive as zeros (their statistics too), which is
    // harmless: P = exp2(0 - 0) = 1 meets dO = 0, and dS = 1 * (0 - 0) = 0.
    constexpr int NCH = D / 8, RPL = 64 / NCH, NLD = 64 / RPL / 4;
    unsigned voff[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int row = (4 * i + wave) * RPL + lane / NCH;
        const int pc = lane % NCH;
        const int sw = (D == 128) ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
        voff[i] = (unsigned)row * (unsigned)(Nq * 2) + (unsigned)((pc ^ sw) << 4);
    }
    auto issue_q = [&](int step, int stage) __attribute__((always_inline)) {
        const unsigned sq = lds0 + stage * STAGE;
        const unsigned base = (unsigned)(step * 64) * (unsigned)(Nq * 2);
#pragma unroll
        for (int i = 0; i < NLD; ++i) dma16(__builtin_amdgcn_readfirstlane(sq + (4 * i + wave) * 1024), rsQ, base + voff[i]);
#pragma unroll
        for (int i = 0; i < NLD; ++i) dma16(__builtin_amdgcn_readfirstlane(sq + TILE + (4 * i + wave) * 1024), rsO, base + voff[i]);
        // row statistics of the 64 queries (every wave issues the same two loads, which keeps the
        // number of loads per wave and step equal)
        const unsigned off = (unsigned)(step * 64 + lane) * 4u;
        dma4(sq + 2 * TILE, rsL, off);
        dma4(sq + 2 * TILE + 256, rsD, off);
    };
    constexpr int LPS = 2 * NLD + 2;                // loads per wave and step

    // ---- the pipeline.  The query rows go by in HALVES of 32 (two per 64-row step / LDS stage).  A
    // half n needs three kinds of work: A(n) = S and dP (2*KS MFMAs against the wave's K and V
    // fragments), B(n) = P and dS from them (vector ALU: exp2, mask, products, packing), C(n) = dV and
    // dK (4*NT MFMAs).  A wave runs alone on its SIMD, so nothing overlaps unless the instruction
    // stream interleaves it: ITERATION t issues A(t+1), B(t) and C(t-1) together, one softmax value
    // (two at d = 64) and the LDS reads of a later slot between two MFMA pairs, so that in the steady
    // state the matrix core runs back to back while the exponentials of the half before and the
    // fragment reads of the slots ahead proceed under it.  Fragment reads go through a ring of four
    // register pairs and are issued three slots ahead of their MFMAs, across iteration boundaries
    // too (the LDS answers a read in a few hundred cycles when four waves keep it busy; a single slot
    // of lookahead left every MFMA pair waiting for it).
    // A slot = one MFMA pair: A slot ks = {S += Qfrag * K[ks], dP += dOfrag * V[ks]}; C slot c =
    // {dK[nt] += dS[j] * Qtokens, dV[nt] += P[j] * dOtokens}, j = c / NT, nt = c % NT.
    // Iterations come in pairs (even t = 2s, odd t = 2s+1) so that stage halves are compile-time.  In
    // the even iteration all C slots come first (with a third of the A slots between them): after
    // them no wave reads stage s-1 any more, so ONE barrier there both frees that stage for the loads
    // of step s+3 and publishes step s+1 (awaited just before it), whose rows the odd iteration's A
    // slots read.  Accumulation order of every output element is that of a plain loop over the rows.
    constexpr int NP = 2 * KS;                      // slots per iteration (KS A slots, 2*NT = KS C slots)
    constexpr int VPS = 16 / NP;                    // softmax values per slot
    constexpr int LOOK = KS >= 8 ? 3 : 2, RING = 4;     // the reads issued for the next iteration must follow the barrier
    static_assert(2 * NT == KS && NP % RING == 0 && (16 % NP) == 0 && NP - LOOK >= 3 * KS / 2, "slot layout");
    typedef __attribute__((address_space(3))) unsigned char* lds_u8_ptr;
    typedef const __attribute__((address_space(3))) u32x4_t* lds_u4_cptr;
    typedef float f32x4v_t __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(3))) f32x4v_t* lds_f4_cptr;
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8_t;

    f32x16_t st[2], dpt[2];                         // S / dP of the half being accumulated and of the one in B, by parity
    bf16x8_t ap[2][2], ads[2][2];                   // packed P and dS, [half parity][16-query block]
    bf16x8_t op[RING][2];                           // fragment pairs on their way to the MFMAs
    f32x4v_t lqr[2], dqr[2];                        // log2(e)*LSE and D of four queries at a time, two groups in flight
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int v = 0; v < 16; ++v) { st[h2][v] = 0.f; dpt[h2][v] = 0.f; }

    // is position p of an (even / odd) iteration an A slot, and which A or C slot is it
    constexpr auto is_a = [](bool even, int p) constexpr { return dkv_is_a(KS, even, p); };
    constexpr auto slot_index = [](bool even, int p) constexpr { return dkv_slot_index(KS, even, p); };
    // reads of an A slot (row fragments of Q and dO, half hf of the stage at sb) or of a C slot (token
    // fragments) into ring entry r
    auto read_a = [&](unsigned sb, int hf, int ks, int r) __attribute__((always_inline)) {
        const lds_u8_ptr q = reinterpret_cast<lds_u8_ptr>(sb + ra[ks]);
        op[r][0] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<lds_u4_cptr>(q + hf * 32 * (D * 2)));
        op[r][1] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<lds_u4_cptr>(q + (TILE + hf * 32 * (D * 2))));
    };
    auto read_c = [&](unsigned sb, int hf, int c, int r) __attribute__((always_inline)) {
        const int j = c / NT, nt = c % NT;
        const lds_u8_ptr lo = reinterpret_cast<lds_u8_ptr>(sb + ta[nt][0]);
        const lds_u8_ptr hi = reinterpret_cast<lds_u8_ptr>(sb + ta[nt][1]);
        const int off = (hf * 32 + 16 * j) * (D * 2);
        const s16x4_t q0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lo + off));
        const s16x4_t q1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(hi + off));
        const s16x4_t o0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lo + (TILE + off)));
        const s16x4_t o1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(hi + (TILE + off)));
        op[r][0] = __builtin_bit_cast(bf16x8_t, (s16x8_t)__builtin_shufflevector(q0, q1, 0, 1, 2, 3, 4, 5, 6, 7));
        op[r][1] = __builtin_bit_cast(bf16x8_t, (s16x8_t)__builtin_shufflevector(o0, o1, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    // statistics of queries [4*g4, 4*g4 + 4) (+ 4*hh per lane half) of half hf of the stage at sb
    auto read_stats = [&](unsigned sb, int hf, int g4, int buf) __attribute__((always_inline)) {
        const lds_u8_ptr ps = reinterpret_cast<lds_u8_ptr>(sb + 2 * TILE + 16 * hh);
        lqr[buf] = *reinterpret_cast<lds_f4_cptr>(ps + (hf * 32 + 8 * g4) * 4);
        dqr[buf] = *reinterpret_cast<lds_f4_cptr>(ps + (64 + hf * 32 + 8 * g4) * 4);
    };
    // P and dS of value v (query 8*(v/4) + 4*hh + v%4 of half t): lane = key, register = query
    auto soft = [&](int par, int v, int qrow0, auto MASKED) __attribute__((always_inline)) {
        constexpr bool masked = decltype(MASKED)::value != 0;
        const int v4 = v >> 2, e = v & 3;
        const float lv = lqr[v4 & 1][e], dd = dqr[v4 & 1][e];
        float pr = __builtin_amdgcn_exp2f(st[par][v] * scale2 - lv);
        if (masked) {
            const bool ok = kvalid && (qrow0 + 8 * v4 + 4 * hh + e >= jk);
            pr = ok ? pr : 0.f;
        }
        st[par][v] = pr;
        dpt[par][v] = pr * (dpt[par][v] - dd);
        if ((v & 7) == 7) {                          // a 16-query block (8 registers) is complete
            ap[par][v >> 3] = pack8(st[par], v >> 3);
            ads[par][v >> 3] = pack8(dpt[par], v >> 3);
        }
    };
    // One iteration (see above).  KIND 0: steady state; 1: the very first iteration (no half before it:
    // the C slots' MFMAs are left out, their reads are harmless); 2: the drain after the last half
    // (only the C slots' MFMAs).
    auto iteration = [&](auto EVEN_, auto MASKED, auto KIND_, const int s) __attribute__((always_inline)) {
        constexpr bool EVEN = decltype(EVEN_)::value != 0;
        constexpr int KIND = decltype(KIND_)::value;
        constexpr int hfA = EVEN ? 1 : 0, hfB = EVEN ? 0 : 1, hfC = EVEN ? 1 : 0;
        constexpr int parA = EVEN ? 1 : 0, parB = EVEN ? 0 : 1, parC = EVEN ? 1 : 0;    // parity of halves t+1, t, t-1
        const unsigned sbA = lds0 + (unsigned)((EVEN ? s : s + 1) & 3) * STAGE;
        const unsigned sbB = lds0 + (unsigned)(s & 3) * STAGE;
        const unsigned sbC = lds0 + (unsigned)((EVEN ? s + 3 : s) & 3) * STAGE;
        // the iteration after this one (the fragment reads of its first slots are issued here)
        constexpr int hfA_n = EVEN ? 0 : 1, hfB_n = EVEN ? 1 : 0, hfC_n = EVEN ? 0 : 1;
        const unsigned sbA_n = lds0 + (unsigned)((s + 1) & 3) * STAGE;
        const unsigned sbB_n = lds0 + (unsigned)((EVEN ? s : s + 1) & 3) * STAGE;
        const unsigned sbC_n = lds0 + (unsigned)(s & 3) * STAGE;
        const int qrow0 = c0 + (2 * s + (EVEN ? 0 : 1)) * 32;       // compact row of the first query of half t
        static_for<NP>([&](auto P) __attribute__((always_inline)) {
            constexpr int pp = decltype(P)::value;
            if constexpr (EVEN && pp == 3 * KS / 2 && KIND != 2) {
                // every C slot of this iteration has its fragments: nobody reads stage s-1 any more
                wait_vmcnt<LPS>();          // step s+1 has landed; step s+2 may be in flight
                lds_barrier();
                issue_q(s + 3, (s + 3) & 3);
            }
            // fragment reads of the slot LOOK positions ahead
            {
                constexpr int q = pp + LOOK;
                if constexpr (q < NP) {
                    if constexpr (is_a(EVEN, q)) read_a(sbA, hfA, slot_index(EVEN, q), q % RING);
                    else read_c(sbC, hfC, slot_index(EVEN, q), q % RING);
                } else if constexpr (KIND != 2) {
                    constexpr int qn = q - NP;
                    if constexpr (is_a(!EVEN, qn)) read_a(sbA_n, hfA_n, slot_index(!EVEN, qn), q % RING);
                    else read_c(sbC_n, hfC_n, slot_index(!EVEN, qn), q % RING);
                }
            }
            if constexpr (KIND != 2) {
                // The A-slot MFMAs are inline assembly (see below), so the compiler does not know that the S and dP
                // values which the previous iteration's last A slot produced may still be on their way when this
                // iteration's first softmax value reads them: eight wait states here, on top of the reads above,
                // cover the eleven that an 8-pass MFMA needs ahead of a vector ALU read of its destination.
                if constexpr (pp == 0) asm volatile("s_nop 7");
                // softmax values of half t, with the statistics of the next four queries fetched one group ahead
#pragma unroll
                for (int e = 0; e < VPS; ++e) {
                    const int v = pp * VPS + e;
                    if ((v & 3) == 0) {
                        if (v < 12) read_stats(sbB, hfB, (v >> 2) + 1, ((v >> 2) + 1) & 1);
                        else read_stats(sbB_n, hfB_n, 0, 0);
                    }
                    soft(parB, v, qrow0, MASKED);
                }
            }
            CF_SCHED_FENCE();
            if constexpr (is_a(EVEN, pp)) {
                if constexpr (KIND != 2) {
                    constexpr int ks = slot_index(EVEN, pp);
                    // Inline assembly keeps S and dP in the VGPR file, where the softmax arithmetic reads them:
                    // with the builtin the register allocator accumulates them in AGPRs and copies all 32
                    // registers of a half out again, one v_accvgpr_read each.  The price is that the compiler
                    // no longer sees these MFMAs' latency (see the wait states at the head of an iteration).
                    if constexpr (ks == 0) {
                        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(st[parA]) : "v"(op[pp % RING][0]), "v"(kf[ks]));
                        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(dpt[parA]) : "v"(op[pp % RING][1]), "v"(vf[ks]));
                    } else {
                        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(st[parA]) : "v"(op[pp % RING][0]), "v"(kf[ks]));
                        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(dpt[parA]) : "v"(op[pp % RING][1]), "v"(vf[ks]));
                    }
                }
            } else {
                if constexpr (KIND != 1) {
                    constexpr int c = slot_index(EVEN, pp), j = c / NT, nt = c % NT;
                    dk[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ads[parC][j], op[pp % RING][0], dk[nt], 0, 0, 0);
                    dv[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap[parC][j], op[pp % RING][1], dv[nt], 0, 0, 0);
                }
            }
            CF_SCHED_FENCE();
        });
    };

    // The block walks through HP query heads of its KV group one after the other: the K and V fragments
    // and the dK / dV accumulators stay in registers, only the Q / dO / statistics stream changes, so
    // the group's sum over these heads costs no partial buffer and a tile's fixed costs (fragment fetch,
    // write-out) are paid once per HP heads.
    for (int hi = 0; hi < HP; ++hi) {
    open_head(h0 + hi);
    if (hi > 0) lds_barrier();                      // every wave is done with the previous head's stages
    // Ring of four stages: the loads of step s+3 are issued in pair s, into the stage that step s-1
    // used.  Steps past the end are issued as well (every row out of range: zero fill), so the number
    // of loads in flight is the same in every pair.
    issue_q(0, 0);
    issue_q(1, 1);
    issue_q(2, 2);
    // Everything is waited for here, not only stage 0: the K and V fragments above come from ordinary
    // loads, and as long as the compiler cannot see them completed ahead of the loop it guards their
    // first use inside the loop with a wait of its own, which the hardware applies to the loads just
    // issued as well: every pair would then wait out a whole global-memory latency.
    wait_vmcnt<0>();
    lds_barrier();
    // head: A(0), then the statistics group and the fragment reads that the first iteration starts with
    {
        f32x16_t z;
#pragma unroll
        for (int v = 0; v < 16; ++v) z[v] = 0.f;
        st[0] = z;
        dpt[0] = z;
        static_for<KS>([&](auto K_) __attribute__((always_inline)) {
            constexpr int ks = decltype(K_)::value;
            read_a(lds0, 0, ks, ks % RING);
            st[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[ks % RING][0], kf[ks], st[0], 0, 0, 0);
            dpt[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[ks % RING][1], vf[ks], dpt[0], 0, 0, 0);
        });
        read_stats(lds0, 0, 0, 0);
        static_for<LOOK>([&](auto Q_) __attribute__((always_inline)) {
            constexpr int q = decltype(Q_)::value;
            if constexpr (is_a(true, q)) read_a(lds0, 1, slot_index(true, q), q % RING);
            else read_c(lds0 + 3 * STAGE, 1, slot_index(true, q), q % RING);      // a half that does not exist: never used
        });
        CF_SCHED_FENCE();
    }
    // MASKED: the pair may hold queries that lie before some of the tile's keys (the first two steps
    // of a tile) or the tile has fewer than 128 keys; every later pair of a full tile sees all of its
    // keys and spends no instruction on the mask.
    const int masked_steps = keys_in_tile < 128 ? steps : min(steps, 2);
    iteration(ic<1>{}, ic<1>{}, ic<1>{}, 0);
    iteration(ic<0>{}, ic<1>{}, ic<0>{}, 0);
    int s = 1;
    for (; s < masked_steps; ++s) {
        iteration(ic<1>{}, ic<1>{}, ic<0>{}, s);
        iteration(ic<0>{}, ic<1>{}, ic<0>{}, s);
    }
    for (; s < steps; ++s) {
        iteration(ic<1>{}, ic<0>{}, ic<0>{}, s);
        iteration(ic<0>{}, ic<0>{}, ic<0>{}, s);
    }
    iteration(ic<1>{}, ic<0>{}, ic<2>{}, steps);     // drain: C of the last half
    wait_vmcnt<0>();                                // the zero-fill loads of the steps past the end
    }

    if (G == HP) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = wave * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
                if (r < keys_in_tile) {
                    const int64_t off = (int64_t)(c0 + r) * Nkv + g * D + nt * 32 + slot;
                    p.dk_kept[off] = f32_to_bf16(dk[nt][v] * p.scale);
                    p.dv_kept[off] = f32_to_bf16(dv[nt][v]);
                }
            }
        }
    } else {
        const int64_t part = (int64_t)((h0 - g * G) / HP) * p.n_kept * Nkv;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = wave * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
                if (r < keys_in_tile) {
                    const int64_t off = part + (int64_t)(c0 + r) * Nkv + g * D + nt * 32 + slot;
                    p.dk_part[off] = dk[nt][v];
                    p.dv_part[off] = dv[nt][v];
                }
            }
        }
    }
}

// dk = scale * sum_g dk_part[g], dv = sum_g dv_part[g]   (fixed order: deterministic)
__global__ __launch_bounds__(256) void attn_dkv_reduce_kernel(const float* __restrict__ dk_part,
                                                              const float* __restrict__ dv_part, int Hq, int Hkv,
                                                              int n_cu, int n_max, const int32_t* __restrict__ n_dev,
                                                              int Nkv, float scale,
                                                              bf16_t* __restrict__ dk, bf16_t* __restrict__ dv) {
    const int n_live = live_rows(n_max, n_dev);
    const int hp = attn_heads_per_block(n_live, Hq, Hq / Hkv, n_cu);
    const int G = Hq / Hkv / hp;                                        // partials per KV group
    if (G == 1) return;                                                 // the dK/dV blocks wrote the results themselves
    const int64_t n_elems = (int64_t)n_max * Nkv;                       // stride between two partials
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i >= (int64_t)n_live * Nkv) return;
    float sk[8], sv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { sk[e] = 0.f; sv[e] = 0.f; }
    for (int g = 0; g < G; ++g) {
        const float4* pk = reinterpret_cast<const float4*>(dk_part + (int64_t)g * n_elems + i);
        const float4* pv = reinterpret_cast<const float4*>(dv_part + (int64_t)g * n_elems + i);
        const float4 a0 = pk[0], a1 = pk[1], b0 = pv[0], b1 = pv[1];
        sk[0] += a0.x; sk[1] += a0.y; sk[2] += a0.z; sk[3] += a0.w;
        sk[4] += a1.x; sk[5] += a1.y; sk[6] += a1.z; sk[7] += a1.w;
        sv[0] += b0.x; sv[1] += b0.y; sv[2] += b0.z; sv[3] += b0.w;
        sv[4] += b1.x; sv[5] += b1.y; sv[6] += b1.z; sv[7] += b1.w;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) sk[e] *= scale;
    Vec<bf16_t>::store(dk + i, sk);
    Vec<bf16_t>::store(dv + i, sv);
}

// stat[0][h][j] = log2(e) * LSE(b, h, position of kept row j); stat[1][h][j] = D = sum_c dO*O of
// (row j, head h): the row terms of the FlashAttention backward, laid out so that the 64 rows a
// dK/dV block needs per step are contiguous.  d/8 lanes share one (row, head).
// o_full / q_full (nullable, need idx): the attention output and the queries are still stored full
// length; the pass reads their kept rows through idx and writes the compact copies o_out / q_out
// that the parameter-gradient GEMM of the output projection and the attention kernels' tile loads
// use (the gathers of the two tensors folded into this read).
__global__ __launch_bounds__(256) void attn_stats_kernel(const bf16_t* __restrict__ do_kept,
                                                         const bf16_t* __restrict__ o_rows,
                                                         const float* __restrict__ lse_full,
                                                         const int32_t* __restrict__ idx, int n_max,
                                                         const int32_t* __restrict__ n_dev,
                                                         int Hq, int d, int S, float* __restrict__ stat,
                                                         const bf16_t* __restrict__ o_full, bf16_t* __restrict__ o_out,
                                                         const bf16_t* __restrict__ q_full, bf16_t* __restrict__ q_out) {
    const int n_kept = live_rows(n_max, n_dev);
    const int lanes = d / 8;
    const int64_t total = (int64_t)n_kept * Hq * lanes;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    float s = 0.f;
    const int64_t pair = gid / lanes;
    if (gid < total) {
        const int part = (int)(gid % lanes);
        float a[8], b[8];
        Vec<bf16_t>::load(do_kept + pair * d + part * 8, a);
        if (o_full != nullptr) {
            const int64_t src = ((int64_t)idx[pair / Hq] * Hq + pair % Hq) * d + part * 8;
            const uint4 ov = *reinterpret_cast<const uint4*>(o_full + src);
            *reinterpret_cast<uint4*>(o_out + pair * d + part * 8) = ov;
            if (q_full != nullptr)
                *reinterpret_cast<uint4*>(q_out + pair * d + part * 8) = *reinterpret_cast<const uint4*>(q_full + src);
            const unsigned w[4] = {ov.x, ov.y, ov.z, ov.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                b[2 * i] = __uint_as_float(w[i] << 16);
                b[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
            }
        } else {
            Vec<bf16_t>::load(o_rows + pair * d + part * 8, b);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) s += a[e] * b[e];
    }
    for (int o = lanes >> 1; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (gid < total && (gid % lanes) == 0) {
        const int j = (int)(pair / Hq), h = (int)(pair % Hq);
        const int64_t tok = idx ? idx[j] : j;
        const int64_t bb = tok / S, pos = tok - bb * S;
        stat[(int64_t)h * n_max + j] = lse_full[(bb * Hq + h) * S + pos] * LOG2E;
        stat[(int64_t)(Hq + h) * n_max + j] = s;
    }
}

bool attn_mfma_supported(const cf_layer_desc& L) {
    return L.dtype == CF_BF16 && (L.d == 64 || L.d == 128);
}

// bytes of fp32 per-head partials behind the D row statistics (0 for MHA)
size_t attn_mfma_partial_bytes(const cf_layer_desc& L, int n_kept) {
    if (!attn_mfma_supported(L) || L.Hq == L.Hkv) return 0;
    return align_up((size_t)2 * (size_t)(n_kept > 0 ? n_kept : 1) * L.Hq * L.d * sizeof(float), 256);
}

template <int D>
static hipError_t launch_t(const AttnParams& p, const bf16_t* o_rows, const float* lse_full, float* stat,
                           const bf16_t* o_full, bf16_t* o_out, const bf16_t* q_full, bf16_t* q_out, hipStream_t st) {
    constexpr int smem_dq = 2 * 2 * 64 * D * 2;
    constexpr int smem_dkv = 4 * (2 * 64 * D * 2 + 512);
    static std::atomic<uint64_t> lds_ok_dq{0}, lds_ok_dkv{0};
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(&attn_dq_kernel<D>), smem_dq, lds_ok_dq);
    if (e != hipSuccess) return e;
    e = allow_dynamic_lds(reinterpret_cast<const void*>(&attn_dkv_kernel<D>), smem_dkv, lds_ok_dkv);
    if (e != hipSuccess) return e;
    const int n_kept = p.n_kept;        // grids cover the upper bound of the row count
    {
        const int64_t total = (int64_t)n_kept * p.Hq * (D / 8);
        attn_stats_kernel<<<(int)((total + 255) / 256), 256, 0, st>>>(p.do_kept, o_rows, lse_full, p.idx, n_kept,
                                                                     p.n_dev, p.Hq, D, p.S, stat, o_full, o_out,
                                                                     q_full, q_out);
    }
    const int max_per_seq = n_kept < p.S ? n_kept : p.S;
    const int tiles = ceil_div(max_per_seq, 128);
    attn_dq_kernel<D><<<dim3(p.Hq * p.B, tiles), 256, smem_dq, st>>>(p);
    attn_dkv_kernel<D><<<dim3(p.Hq * p.B * tiles), 256, smem_dkv, st>>>(p);
    if (p.Hq != p.Hkv) {
        const int64_t n_elems = (int64_t)n_kept * p.Hkv * D;
        attn_dkv_reduce_kernel<<<ceil_div(n_elems / 8, 256), 256, 0, st>>>(p.dk_part, p.dv_part, p.Hq, p.Hkv, p.n_cu,
                                                                          n_kept, p.n_dev, p.Hkv * D, p.scale,
                                                                          p.dk_kept, p.dv_kept);
    }
    return hipGetLastError();
}

// o_full / q_full (both nullable, need idx): attention output and queries at full length; their kept
// rows are then copied to o_kept / q_kept (which must be writable buffers) by the row-statistics pass.
hipError_t launch_attn_bwd_mfma(const cf_layer_desc& L, float scale, const void* q_kept,
                                const void* k_full, const void* v_full, const void* o_kept,
                                const float* lse_full, const void* do_kept, float* stat,
                                const int32_t* idx, const int32_t* cu_kept, RowCount rows, void* dq_kept,
                                void* dk_kept, void* dv_kept, float* partials, hipStream_t st,
                                const void* o_full, const void* q_full) {
    AttnParams p;
    const int n_kept = rows.n;
    p.q_kept = (const bf16_t*)q_kept; p.k_full = (const bf16_t*)k_full; p.v_full = (const bf16_t*)v_full;
    p.do_kept = (const bf16_t*)do_kept; p.stat = stat; p.idx = idx;
    p.cu_kept = cu_kept; p.dq_kept = (bf16_t*)dq_kept; p.dk_kept = (bf16_t*)dk_kept;
    p.dv_kept = (bf16_t*)dv_kept; p.B = L.B; p.S = L.S; p.Hq = L.Hq; p.Hkv = L.Hkv; p.scale = scale;
    p.n_kept = n_kept;
    p.n_cu = compute_units();
    p.n_dev = rows.dev;
    p.dk_part = partials;
    p.dv_part = partials ? partials + (size_t)n_kept * L.Hq * L.d : nullptr;
    bf16_t* o_out = o_full ? (bf16_t*)const_cast<void*>(o_kept) : nullptr;
    bf16_t* q_out = q_full ? (bf16_t*)const_cast<void*>(q_kept) : nullptr;
    if (L.d == 64)
        return launch_t<64>(p, (const bf16_t*)o_kept, lse_full, stat, (const bf16_t*)o_full, o_out,
                            (const bf16_t*)q_full, q_out, st);
    return launch_t<128>(p, (const bf16_t*)o_kept, lse_full, stat, (const bf16_t*)o_full, o_out,
                         (const bf16_t*)q_full, q_out, st);
}

}  // namespace cf
