// Filtered attention backward on the matrix cores (Sec. 3.1, Eq. 3-4), bf16 in,
// fp32 softmax statistics and accumulators.  Two deterministic kernels, no atomics:
//
//   dQ kernel   (Eq. 3 dS*K-hat + Eq. 4 dS*K-check in one pass): a block owns 128
//               kept queries of one (sequence, query head) and walks over ALL key
//               tiles up to the last query's original position; P is rebuilt
//               from the saved LSE, so filtered keys contribute exactly as in
//               the forward pass.
//   dK/dV kernel (Eq. 3): a block owns 128 KEPT keys of one (sequence, KV head) and
//               walks over the kept queries at or after them, for every query
//               head of the group; rows of filtered tokens are never formed.
//               Kept rows are in position order, so causality is "compact query
//               index >= compact key index".
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

namespace cf {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;

static constexpr float LOG2E = 1.4426950408889634f;

struct AttnParams {
    const bf16_t *q_kept, *k_full, *v_full, *do_kept;
    const float *lse_full, *Drow;
    const int32_t *idx, *cu_kept;
    bf16_t *dq_kept, *dk_kept, *dv_kept;
    int B, S, Hq, Hkv;
    float scale;
};

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

// ---------------------------------------------------------------------------
// dQ kernel
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_dq_kernel(AttnParams p) {
    constexpr int NCH = D / 8, KS = D / 16, NT = D / 32;
    constexpr int TILE = 64 * D * 2;            // one 64-token tile in bytes
    constexpr int LD = 64 * NCH / 256;          // 16-byte chunks per thread per tile
    extern __shared__ __align__(16) unsigned char smem[];   // [2 stages][K tile, V tile]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slot = lane & 31, hh = lane >> 5;
    const int b = blockIdx.z, h = blockIdx.y, g = h / (p.Hq / p.Hkv);
    const int Nq = p.Hq * D, Nkv = p.Hkv * D;
    const int seq_begin = p.cu_kept ? p.cu_kept[b] : b * p.S;
    const int seq_end = p.cu_kept ? p.cu_kept[b + 1] : (b + 1) * p.S;
    const int cnt = seq_end - seq_begin;
    const int qt = gridDim.x - 1 - blockIdx.x;        // heaviest (latest) query tiles first
    if (qt * 128 >= cnt) return;
    const int j0 = seq_begin + qt * 128;
    const int rows_in_tile = min(128, cnt - qt * 128);

    // this lane's query
    const int jq = j0 + wave * 32 + slot;
    const bool qvalid = wave * 32 + slot < rows_in_tile;
    const int pos = qvalid ? (p.idx ? p.idx[jq] : jq) - b * p.S : -1;
    const float lse2 = qvalid ? p.lse_full[((int64_t)b * p.Hq + h) * p.S + pos] * LOG2E : 0.f;
    const float Dq = qvalid ? p.Drow[(int64_t)jq * p.Hq + h] : 0.f;
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
    int wave_maxpos = -1;
    {
        const int wrows = min(32, rows_in_tile - wave * 32);
        if (wrows > 0) {
            const int jw = j0 + wave * 32 + wrows - 1;
            wave_maxpos = (p.idx ? p.idx[jw] : jw) - b * p.S;
        }
    }
    const float scale2 = p.scale * LOG2E;

    f32x16_t acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nt][v] = 0.f;

    uint4 rk[LD], rv[LD];
    auto load_kv = [&](int kt) {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int q = tid + 256 * i;
            const int row = q / NCH, c = q % NCH;
            const int key = kt * 64 + row;
            if (key <= maxpos) {
                const int64_t off = ((int64_t)b * p.S + key) * Nkv + g * D + c * 8;
                rk[i] = *reinterpret_cast<const uint4*>(p.k_full + off);
                rv[i] = *reinterpret_cast<const uint4*>(p.v_full + off);
            } else {
                rk[i] = make_uint4(0, 0, 0, 0);
                rv[i] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_kv = [&](int stage) {
        unsigned char* sk = smem + stage * 2 * TILE;
        unsigned char* sv = sk + TILE;
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int q = tid + 256 * i;
            const int off = tile_off<D>(q / NCH, q % NCH);
            *reinterpret_cast<uint4*>(sk + off) = rk[i];
            *reinterpret_cast<uint4*>(sv + off) = rv[i];
        }
    };

    load_kv(0);
    store_kv(0);
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nkt;
        if (more) load_kv(kt + 1);
        if (kt * 64 <= wave_maxpos) {
            const unsigned char* sk = smem + cur * 2 * TILE;
            const unsigned char* sv = sk + TILE;
            f32x16_t st[2], dpt[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) { st[mt][v] = 0.f; dpt[mt][v] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    st[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_rows<D>(sk, mt * 32 + slot, ks, hh), qf[ks], st[mt], 0, 0, 0);
                    dpt[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_rows<D>(sv, mt * 32 + slot, ks, hh), dof[ks], dpt[mt], 0, 0, 0);
                }
            }
            // dS^T = P^T o (dP^T - D): lane = query, register = key
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = kt * 64 + mt * 32 + 8 * (v >> 2) + 4 * hh + (v & 3);
                    const float pr = key <= pos ? __builtin_amdgcn_exp2f(st[mt][v] * scale2 - lse2) : 0.f;
                    st[mt][v] = pr * (dpt[mt][v] - Dq);
                }
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const bf16x8_t a = pack8(st[mt], j);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            a, frag_tokens<D>(sk, mt * 32 + 16 * j, nt, lane), acc[nt], 0, 0, 0);
                }
            }
        }
        if (more) store_kv(cur ^ 1);
        __syncthreads();
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
// dK/dV kernel
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_dkv_kernel(AttnParams p) {
    constexpr int NCH = D / 8, KS = D / 16, NT = D / 32;
    constexpr int TILE = 64 * D * 2;
    constexpr int LD = 64 * NCH / 256;
    constexpr int STAGE = 2 * TILE + 512;       // Q tile, dO tile, lse2[64], D[64]
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slot = lane & 31, hh = lane >> 5;
    const int b = blockIdx.z, g = blockIdx.y, G = p.Hq / p.Hkv;
    const int Nq = p.Hq * D, Nkv = p.Hkv * D;
    const int seq_begin = p.cu_kept ? p.cu_kept[b] : b * p.S;
    const int seq_end = p.cu_kept ? p.cu_kept[b + 1] : (b + 1) * p.S;
    const int cnt = seq_end - seq_begin;
    const int kt = blockIdx.x;
    if (kt * 128 >= cnt) return;
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
    const int ntq = (seq_end - c0 + 63) / 64;       // query tiles from the first key to the sequence end
    const int steps = G * ntq;
    const int wave_first_key = c0 + wave * 32;

    f32x16_t dk[NT], dv[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) { dk[nt][v] = 0.f; dv[nt][v] = 0.f; }

    uint4 rq[LD], rdo[LD];
    float rl = 0.f, rd = 0.f;
    auto load_q = [&](int step) {
        const int h = g * G + step / ntq;
        const int qbase = c0 + (step % ntq) * 64;
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int q = tid + 256 * i;
            const int row = qbase + q / NCH, c = q % NCH;
            if (row < seq_end) {
                const int64_t off = (int64_t)row * Nq + h * D + c * 8;
                rq[i] = *reinterpret_cast<const uint4*>(p.q_kept + off);
                rdo[i] = *reinterpret_cast<const uint4*>(p.do_kept + off);
            } else {
                rq[i] = make_uint4(0, 0, 0, 0);
                rdo[i] = make_uint4(0, 0, 0, 0);
            }
        }
        if (tid < 64) {
            const int row = qbase + tid;
            if (row < seq_end) {
                const int pos = (p.idx ? p.idx[row] : row) - b * p.S;
                rl = p.lse_full[((int64_t)b * p.Hq + h) * p.S + pos] * LOG2E;
                rd = p.Drow[(int64_t)row * p.Hq + h];
            } else {
                rl = __builtin_inff();      // exp2(x - inf) = 0 for rows past the sequence end
                rd = 0.f;
            }
        }
    };
    auto store_q = [&](int stage) {
        unsigned char* sq = smem + stage * STAGE;
        unsigned char* sdo = sq + TILE;
        float* sl = reinterpret_cast<float*>(sq + 2 * TILE);
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int q = tid + 256 * i;
            const int off = tile_off<D>(q / NCH, q % NCH);
            *reinterpret_cast<uint4*>(sq + off) = rq[i];
            *reinterpret_cast<uint4*>(sdo + off) = rdo[i];
        }
        if (tid < 64) { sl[tid] = rl; sl[64 + tid] = rd; }
    };

    load_q(0);
    store_q(0);
    __syncthreads();
    for (int step = 0; step < steps; ++step) {
        const int cur = step & 1;
        const bool more = step + 1 < steps;
        if (more) load_q(step + 1);
        const int qbase = c0 + (step % ntq) * 64;
        if (qbase + 63 >= wave_first_key && wave * 32 < keys_in_tile) {
            const unsigned char* sq = smem + cur * STAGE;
            const unsigned char* sdo = sq + TILE;
            const float* sl = reinterpret_cast<const float*>(sq + 2 * TILE);
            f32x16_t st[2], dpt[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) { st[mt][v] = 0.f; dpt[mt][v] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    st[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_rows<D>(sq, mt * 32 + slot, ks, hh), kf[ks], st[mt], 0, 0, 0);
                    dpt[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        frag_rows<D>(sdo, mt * 32 + slot, ks, hh), vf[ks], dpt[mt], 0, 0, 0);
                }
            }
            // P and dS: lane = key, register = query
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const int ql = mt * 32 + 8 * v4 + 4 * hh;
                    const float4 l4 = *reinterpret_cast<const float4*>(sl + ql);
                    const float4 d4 = *reinterpret_cast<const float4*>(sl + 64 + ql);
                    const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
                    const float dd[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = 4 * v4 + e;
                        const bool ok = kvalid && (qbase + ql + e >= jk);
                        const float pr = ok ? __builtin_amdgcn_exp2f(st[mt][v] * scale2 - lv[e]) : 0.f;
                        st[mt][v] = pr;
                        dpt[mt][v] = pr * (dpt[mt][v] - dd[e]);
                    }
                }
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const bf16x8_t ap = pack8(st[mt], j);
                    const bf16x8_t ads = pack8(dpt[mt], j);
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        dv[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            ap, frag_tokens<D>(sdo, mt * 32 + 16 * j, nt, lane), dv[nt], 0, 0, 0);
                        dk[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            ads, frag_tokens<D>(sq, mt * 32 + 16 * j, nt, lane), dk[nt], 0, 0, 0);
                    }
                }
            }
        }
        if (more) store_q(cur ^ 1);
        __syncthreads();
    }

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
}

bool attn_mfma_supported(const cf_layer_desc& L) {
    return L.dtype == CF_BF16 && (L.d == 64 || L.d == 128);
}

template <int D>
static hipError_t launch_t(const AttnParams& p, int n_kept, hipStream_t st) {
    constexpr int smem_dq = 2 * 2 * 64 * D * 2;
    constexpr int smem_dkv = 2 * (2 * 64 * D * 2 + 512);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_dq_kernel<D>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem_dq);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_dkv_kernel<D>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem_dkv);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int max_per_seq = n_kept < p.S ? n_kept : p.S;
    const int tiles = ceil_div(max_per_seq, 128);
    attn_dq_kernel<D><<<dim3(tiles, p.Hq, p.B), 256, smem_dq, st>>>(p);
    attn_dkv_kernel<D><<<dim3(tiles, p.Hkv, p.B), 256, smem_dkv, st>>>(p);
    return hipGetLastError();
}

hipError_t launch_attn_bwd_mfma(const cf_layer_desc& L, float scale, const void* q_kept,
                                const void* k_full, const void* v_full, const float* lse_full,
                                const void* do_kept, const float* Drow, const int32_t* idx,
                                const int32_t* cu_kept, int n_kept, void* dq_kept, void* dk_kept,
                                void* dv_kept, hipStream_t st) {
    AttnParams p;
    p.q_kept = (const bf16_t*)q_kept; p.k_full = (const bf16_t*)k_full; p.v_full = (const bf16_t*)v_full;
    p.do_kept = (const bf16_t*)do_kept; p.lse_full = lse_full; p.Drow = Drow; p.idx = idx;
    p.cu_kept = cu_kept; p.dq_kept = (bf16_t*)dq_kept; p.dk_kept = (bf16_t*)dk_kept;
    p.dv_kept = (bf16_t*)dv_kept; p.B = L.B; p.S = L.S; p.Hq = L.Hq; p.Hkv = L.Hkv; p.scale = scale;
    if (L.d == 64) return launch_t<64>(p, n_kept, st);
    return launch_t<128>(p, n_kept, st);
}

}  // namespace cf
