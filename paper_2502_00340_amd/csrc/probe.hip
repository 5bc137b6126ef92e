// Measurement probes: what this chip sustains when a kernel does nothing but the bound
// operation.  They give the reduced GEMMs (Sec. 3.2) and the gather / row-local kernels a
// MEASURED ceiling next to the published peaks (2.5 PFLOP/s dense bf16, 8 TB/s HBM):
//
//   mfma probe: the GEMM's inner product shape (a 128x128 wave tile = 8 x 8 accumulators of
//               16x16x32 bf16 MFMAs, four waves per block, one block per CU) with every operand
//               resident in registers: no LDS traffic, no global traffic, no address arithmetic.
//               Operands are pseudo-random non-zero values (an all-zero operand draws far less
//               power than real data and overstates the ceiling of a power-limited chip).
//   copy probe: dst[i] = src[i] in 16-byte words, four independent loads in flight per lane,
//               one contiguous 16 KB range per block.
#include "common.h"
#include "mfma_util.h"

namespace cf {

__device__ __forceinline__ unsigned probe_hash(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// eight bf16 values in (-2, 2), none zero, different in every lane and fragment
__device__ __forceinline__ bf16x8_t probe_fragment(unsigned seed) {
    u32x4_t w;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const unsigned h = probe_hash(seed * 4u + e);
        const float lo = ((float)(h & 0xFFFFu) + 1.0f) * (1.0f / 32768.0f) - 1.0f;
        const float hi = ((float)(h >> 16) + 1.0f) * (1.0f / 32768.0f) - 1.0f;
        w[e] = pack_bf16x2(lo == 0.f ? 0.5f : 2.f * lo, hi == 0.f ? -0.5f : 2.f * hi);
    }
    return __builtin_bit_cast(bf16x8_t, w);
}

__global__ __launch_bounds__(256) void mfma_probe_kernel(float* __restrict__ sink, int iters) {
    const unsigned tid = blockIdx.x * 256u + threadIdx.x;
    bf16x8_t a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = probe_fragment(tid * 16u + i);
        b[i] = probe_fragment(tid * 16u + 8u + i);
    }
    f32x4_t acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(b[j]), "v"(a[i]));
    }
    asm volatile("s_nop 15\n\ts_nop 15");        // the last MFMAs' results are still on the way (see gemm.hip)
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[i][j][0] + acc[i][j][3];
    sink[tid] = s;
}

// The same MFMA loop with the GEMM's LDS fragment reads mixed in at the GEMM's ratio: READS 1 = 16
// ds_read_b128 per 64 MFMAs (mode NT), READS 2 = 32 ds_read_b64_tr_b16 per 64 MFMAs (mode TN), every read
// behind an MFMA, nothing waiting for them inside the loop (their results are folded into the sink after
// it).  The LDS holds pseudo-random bf16 values; reads are conflict-free (16 bytes per lane, consecutive).
template <int READS>
__global__ __launch_bounds__(256) void mfma_lds_probe_kernel(float* __restrict__ sink, int iters) {
    __shared__ __align__(16) unsigned lds[16384];
    const unsigned tid = blockIdx.x * 256u + threadIdx.x;
    for (int i = threadIdx.x; i < 16384; i += 256) {
        const unsigned h = probe_hash(i * 2654435761u + blockIdx.x);
        lds[i] = (h & 0x807F807Fu) | 0x3F003F00u;                   // two bf16 values in +-[0.5, 1)
    }
    __syncthreads();
    bf16x8_t a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = probe_fragment(tid * 16u + i);
        b[i] = probe_fragment(tid * 16u + 8u + i);
    }
    f32x4_t acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
    u32x4_t r[4];
    u32x2_t r2[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { r[i] = u32x4_t{0, 0, 0, 0}; r2[i] = u32x2_t{0, 0}; }
    // wave w reads bytes [1024 w + 16 lane + 4096 k, +16), k < 8: inside the 64 KB array
    const unsigned addr = lds_addr_of(lds) + (threadIdx.x & 63) * 16 + (threadIdx.x >> 6) * 1024;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int m = i * 8 + j;
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(b[j]), "v"(a[i]));
                if (READS == 1 && (m & 3) == 1)
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r[(m >> 2) & 3]) : "v"(addr), "n"(((m >> 2) & 7) * 4096));
                if (READS == 2 && (m & 1) == 1)
                    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r2[(m >> 1) & 3]) : "v"(addr), "n"(((m >> 1) & 7) * 4096));
            }
    }
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 15\n\ts_nop 15" ::: "memory");
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += acc[i][j][0] + acc[i][j][3];
    unsigned x = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) x ^= r[i][0] ^ r[i][3] ^ r2[i][0] ^ r2[i][1];
    sink[tid] = s + (float)(x & 0xFF);
}

// block b copies words [b*1024, (b+1)*1024): four loads per lane in flight, then four stores, both with
// the non-temporal hint (the data is touched once).  Of the variants measured on this chip (grid-stride
// loops of 1, 4 or 8 words per lane, with and without the hint, 2 K to 64 K blocks; one, two, four or
// eight words per lane of a block-contiguous range; the runtime's own device-to-device copy) this one
// and its one-word-per-lane form were the fastest.
typedef unsigned int copy_word_t __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void copy_probe_kernel(const copy_word_t* __restrict__ src,
                                                         copy_word_t* __restrict__ dst, size_t n16) {
    const size_t base = (size_t)blockIdx.x * 1024 + threadIdx.x;
    copy_word_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (base + u * 256 < n16) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (base + u * 256 < n16) __builtin_nontemporal_store(v[u], dst + base + u * 256);
}

}  // namespace cf

using namespace cf;

extern "C" {

cf_status cf_probe_mfma_bf16(int32_t n_blocks, int32_t iters, float* sink, double* flops_out, cf_stream stream) {
    if (!sink) return CF_ERR_NULL;
    if (n_blocks <= 0 || n_blocks > 65536 || iters <= 0 || ((uintptr_t)sink % 4) != 0) return CF_ERR_SHAPE;
    mfma_probe_kernel<<<n_blocks, 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(sink, iters);
    if (hipGetLastError() != hipSuccess) return CF_ERR_HIP;
    // 4 waves x 64 MFMAs of 16x16x32 (2*16*16*32 flop) per iteration and block
    if (flops_out) *flops_out = (double)n_blocks * 4.0 * 64.0 * 16384.0 * (double)iters;
    return CF_OK;
}

cf_status cf_probe_mfma_lds_bf16(int32_t n_blocks, int32_t iters, int32_t reads, float* sink, double* flops_out,
                                 cf_stream stream) {
    if (!sink) return CF_ERR_NULL;
    if (n_blocks <= 0 || n_blocks > 65536 || iters <= 0 || reads < 0 || reads > 2 || ((uintptr_t)sink % 4) != 0)
        return CF_ERR_SHAPE;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (reads == 0) mfma_lds_probe_kernel<0><<<n_blocks, 256, 0, st>>>(sink, iters);
    else if (reads == 1) mfma_lds_probe_kernel<1><<<n_blocks, 256, 0, st>>>(sink, iters);
    else mfma_lds_probe_kernel<2><<<n_blocks, 256, 0, st>>>(sink, iters);
    if (hipGetLastError() != hipSuccess) return CF_ERR_HIP;
    if (flops_out) *flops_out = (double)n_blocks * 4.0 * 64.0 * 16384.0 * (double)iters;
    return CF_OK;
}

cf_status cf_probe_copy(const void* src, void* dst, size_t bytes, cf_stream stream) {
    if (!src || !dst) return CF_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || ((uintptr_t)src % 16) != 0 || ((uintptr_t)dst % 16) != 0) return CF_ERR_SHAPE;
    const size_t n16 = bytes / 16;
    const size_t blocks = (n16 + 1023) / 1024;
    if (blocks > 0x7FFFFFFFull) return CF_ERR_UNSUPPORTED;
    copy_probe_kernel<<<(unsigned)blocks, 256, 0, reinterpret_cast<hipStream_t>(stream)>>>(
        static_cast<const copy_word_t*>(src), static_cast<copy_word_t*>(dst), n16);
    return hipGetLastError() == hipSuccess ? CF_OK : CF_ERR_HIP;
}

}  // extern "C"
