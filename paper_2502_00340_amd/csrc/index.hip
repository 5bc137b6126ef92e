// Keep-index build (order-preserving stream compaction of the keep mask) and
// row gather: the "shrink the sequence dimension" step of Sec. 3.2.
#include "common.h"

namespace cf {

static constexpr int IDX_THREADS = 256;
static constexpr int IDX_PER_THREAD = 16;
static constexpr int IDX_CHUNK = IDX_THREADS * IDX_PER_THREAD;   // tokens per block
static constexpr int IDX_SELF_COUNT_MAX_BLOCKS = 8;

// number of non-zero bytes among 16 mask bytes starting at t0 (bytes >= T read as 0)
__device__ __forceinline__ void load_flags(const uint8_t* mask, int64_t t0, int64_t T, bool aligned,
                                           unsigned (&w)[4]) {
    if (aligned && t0 + 16 <= T) {
        uint4 v = *reinterpret_cast<const uint4*>(mask + t0);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else {
        w[0] = w[1] = w[2] = w[3] = 0u;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            int64_t t = t0 + e;
            unsigned b = (t < T) ? mask[t] : 0u;
            w[e >> 2] |= b << (8 * (e & 3));
        }
    }
}

// per byte: 1 if the byte is non-zero
__device__ __forceinline__ unsigned nonzero_bytes(unsigned w) {
    unsigned t = (w | (w >> 4)) & 0x0F0F0F0Fu;
    t = (t | (t >> 2));
    t = (t | (t >> 1)) & 0x01010101u;
    return t;
}

__device__ __forceinline__ int count_flags(const unsigned (&w)[4]) {
    return __popc(nonzero_bytes(w[0])) + __popc(nonzero_bytes(w[1])) +
           __popc(nonzero_bytes(w[2])) + __popc(nonzero_bytes(w[3]));
}

__device__ __forceinline__ int block_sum_256(int v, int* red) {
    // red: 4 ints of LDS
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// Masks of a handful of chunks (up to IDX_SELF_COUNT_MAX_BLOCKS, i.e. every layer-sized batch): one
// launch, no scratch; every block counts the mask bytes before its chunk itself.
__global__ __launch_bounds__(IDX_THREADS) void mask_scatter_kernel(
    const uint8_t* __restrict__ mask, int64_t T, int S, int B, int aligned,
    int32_t* __restrict__ idx, int32_t* __restrict__ cu_kept, int32_t* __restrict__ n_kept_dev) {
    __shared__ int red[4];
    __shared__ int wave_tot[4];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    int base;
    {
        int before = 0;
        unsigned w[4];
        for (int c = 0; c < (int)blockIdx.x; ++c) {
            load_flags(mask, (int64_t)c * IDX_CHUNK + (int64_t)tid * IDX_PER_THREAD, T, aligned != 0, w);
            before += count_flags(w);
        }
        base = block_sum_256(before, red);
    }

    unsigned w[4];
    const int64_t t0 = (int64_t)blockIdx.x * IDX_CHUNK + (int64_t)tid * IDX_PER_THREAD;
    load_flags(mask, t0, T, aligned != 0, w);
    const int cnt = count_flags(w);

    // exclusive scan of cnt over the block: wave scan, then wave totals
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(incl, o, 64);
        if (lane >= o) incl += n;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int wave_base = 0;
    for (int i = 0; i < wave; ++i) wave_base += wave_tot[i];
    int pos = base + wave_base + incl - cnt;

    if (t0 < T) {
        int s = (int)(t0 % S);
        int b = (int)(t0 / S);
#pragma unroll
        for (int e = 0; e < IDX_PER_THREAD; ++e) {
            int64_t t = t0 + e;
            if (t < T) {
                if (s == 0) cu_kept[b] = pos;
                if ((w[e >> 2] >> (8 * (e & 3))) & 0xFFu) idx[pos++] = (int32_t)t;
                if (++s == S) { s = 0; ++b; }
            }
        }
        if (t0 + IDX_PER_THREAD >= T) {   // this thread owns token T-1
            cu_kept[B] = pos;
            if (n_kept_dev != nullptr) *n_kept_dev = pos;
        }
    }
}

// ---------------------------------------------------------------------------
// Masks of more than a handful of chunks: two launches over SPANS of IDX_SPAN_CHUNKS chunks (8192
// tokens), one block per span.  The first counts the kept tokens of every span; the second has every block add up the counts of the spans before its own
// (two thousand numbers for 16 M tokens, read by all threads at once: no scan kernel, no waiting on
// other blocks) and then compact its span chunk by chunk: flags -> wave / block scan -> the chunk's
// kept positions gathered in LDS -> full 256-byte lines out.  The second pass over the mask finds it
// in the memory-side cache.
// (A single-pass chained scan with decoupled look-back was measured as well: one status word per chunk
// has to cross from one XCD's L2 to another's through memory, about a microsecond per hop, and the chain
// of hops made it slower than the two launches: 70 us against 45 us for 16 M tokens.)
// ---------------------------------------------------------------------------
static constexpr int IDX_SPAN_CHUNKS = 2;
static constexpr int64_t IDX_SPAN = (int64_t)IDX_SPAN_CHUNKS * IDX_CHUNK;

__global__ __launch_bounds__(IDX_THREADS) void mask_span_count_kernel(const uint8_t* __restrict__ mask, int64_t T,
                                                                      int aligned, int32_t* __restrict__ span_count) {
    __shared__ int red[4];
    const int64_t s0 = (int64_t)blockIdx.x * IDX_SPAN + (int64_t)threadIdx.x * IDX_PER_THREAD;
    unsigned w[IDX_SPAN_CHUNKS][4];
#pragma unroll
    for (int c = 0; c < IDX_SPAN_CHUNKS; ++c) load_flags(mask, s0 + (int64_t)c * IDX_CHUNK, T, aligned != 0, w[c]);
    int n = 0;
#pragma unroll
    for (int c = 0; c < IDX_SPAN_CHUNKS; ++c) n += count_flags(w[c]);
    const int total = block_sum_256(n, red);
    if (threadIdx.x == 0) span_count[blockIdx.x] = total;
}

__global__ __launch_bounds__(IDX_THREADS) void mask_span_scatter_kernel(
    const uint8_t* __restrict__ mask, int64_t T, int S, int B, int aligned,
    const int32_t* __restrict__ span_count, int32_t* __restrict__ idx, int32_t* __restrict__ cu_kept,
    int32_t* __restrict__ n_kept_dev) {
    __shared__ int red[4];
    __shared__ int wave_tot[4];
    __shared__ int32_t staged[IDX_CHUNK];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // the span's mask bytes are requested first: they are on their way while the counts are added up
    unsigned wall[IDX_SPAN_CHUNKS][4];
#pragma unroll
    for (int c = 0; c < IDX_SPAN_CHUNKS; ++c)
        load_flags(mask, (int64_t)blockIdx.x * IDX_SPAN + (int64_t)c * IDX_CHUNK + (int64_t)tid * IDX_PER_THREAD, T,
                   aligned != 0, wall[c]);
    int before = 0;
    for (int i = tid; i < (int)blockIdx.x; i += IDX_THREADS) before += span_count[i];
    int base = block_sum_256(before, red);          // kept tokens in all spans before this one

#pragma unroll
    for (int c = 0; c < IDX_SPAN_CHUNKS; ++c) {
        const int64_t t0 = (int64_t)blockIdx.x * IDX_SPAN + (int64_t)c * IDX_CHUNK + (int64_t)tid * IDX_PER_THREAD;
        if ((int64_t)blockIdx.x * IDX_SPAN + (int64_t)c * IDX_CHUNK >= T) break;         // uniform: past the mask's end
        const unsigned (&w)[4] = wall[c];
        const int cnt = count_flags(w);
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int n = __shfl_up(incl, o, 64);
            if (lane >= o) incl += n;
        }
        __syncthreads();                            // the previous chunk's staged positions and totals have been read
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int wave_base = 0;
        for (int i = 0; i < wave; ++i) wave_base += wave_tot[i];
        const int total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
        int pos = wave_base + incl - cnt;           // kept tokens of this chunk before this thread's 16
        if (t0 < T) {
            // T <= 2^30: token numbers fit 32 bits.  Sequence starts inside these 16 tokens (none, as a rule:
            // only then is the division's result used) get their prefix count; bytes past T were read as zero.
            const unsigned u0 = (unsigned)t0;
            unsigned b = (u0 + (unsigned)S - 1u) / (unsigned)S;          // first sequence that starts at or after u0
            unsigned next_start = b * (unsigned)S;
#pragma unroll
            for (int e = 0; e < IDX_PER_THREAD; ++e) {
                const unsigned t = u0 + e;
                if (t == next_start && t < (unsigned)T) {
                    cu_kept[b] = base + pos;
                    ++b;
                    next_start += (unsigned)S;
                }
                if ((w[e >> 2] >> (8 * (e & 3))) & 0xFFu) staged[pos++] = (int32_t)t;
            }
            if (t0 + IDX_PER_THREAD >= T) {         // this thread owns token T-1
                cu_kept[B] = base + pos;
                if (n_kept_dev != nullptr) *n_kept_dev = base + pos;
            }
        }
        __syncthreads();
        for (int i = tid; i < total; i += IDX_THREADS) idx[base + i] = staged[i];
        base += total;
    }
}

size_t index_ws_bytes(int64_t n_tokens) {
    int64_t nspan = (n_tokens + IDX_SPAN - 1) / IDX_SPAN;
    if (nspan < 1) nspan = 1;
    return align_up((size_t)nspan * sizeof(int32_t), 256);      // one count per span
}

hipError_t launch_keep_index(const uint8_t* mask, int B, int S, int32_t* idx, int32_t* cu_kept,
                             int32_t* n_kept_dev, void* ws, hipStream_t st) {
    const int64_t T = (int64_t)B * S;
    const int nblk = ceil_div(T, IDX_CHUNK);
    const int aligned = ((uintptr_t)mask % 16 == 0) ? 1 : 0;
    if (nblk <= IDX_SELF_COUNT_MAX_BLOCKS) {
        mask_scatter_kernel<<<nblk, IDX_THREADS, 0, st>>>(mask, T, S, B, aligned, idx, cu_kept, n_kept_dev);
    } else {
        const int nspan = ceil_div(T, IDX_SPAN);
        int32_t* span_count = static_cast<int32_t*>(ws);
        mask_span_count_kernel<<<nspan, IDX_THREADS, 0, st>>>(mask, T, aligned, span_count);
        mask_span_scatter_kernel<<<nspan, IDX_THREADS, 0, st>>>(mask, T, S, B, aligned, span_count, idx, cu_kept,
                                                                n_kept_dev);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// The same index build for callers that cannot allocate or hand in a workspace: the per-block
// counts live in a file-scope device array.  Every GPU holds its own copy of the array at its own
// address; host code never uses the array's name as a pointer but looks its address up once per
// device (with that device current) and passes that pointer to the kernels.  The kernels write
// every entry they later read (span b's count, b < number of spans), so nothing has to be cleared
// between calls; calls that overlap on one GPU share the array and race.
// ---------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[IDX_STATIC_MAX_TOKENS / IDX_SPAN];

hipError_t launch_keep_index_static(const uint8_t* mask, int B, int S, int32_t* idx, int32_t* cu_kept,
                                    int32_t* n_kept_dev, hipStream_t st) {
    static std::atomic<void*> scratch_ptr[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    void* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    return launch_keep_index(mask, B, S, idx, cu_kept, n_kept_dev, ptr, st);
}

// ---------------------------------------------------------------------------
// gather: dst[j,:] = src[idx[j],:], rows copied as 16-byte (or 4-byte) words
// ---------------------------------------------------------------------------

template <typename W>
__global__ __launch_bounds__(256) void gather_rows_kernel(const W* __restrict__ src,
                                                          const int32_t* __restrict__ idx,
                                                          int n_max, const int32_t* __restrict__ n_dev,
                                                          int words_per_row,
                                                          int lanes_per_row, int rows_per_block,
                                                          W* __restrict__ dst) {
    const int n_rows = live_rows(n_max, n_dev);
    const int r = threadIdx.x / lanes_per_row;
    const int c0 = threadIdx.x % lanes_per_row;
    const int j = blockIdx.x * rows_per_block + r;
    if (r >= rows_per_block || j >= n_rows) return;
    const W* s = src + (int64_t)idx[j] * words_per_row;
    W* d = dst + (int64_t)j * words_per_row;
    for (int c = c0; c < words_per_row; c += lanes_per_row) d[c] = s[c];
}

hipError_t launch_gather(const void* src, int64_t cols_bytes, const int32_t* idx, RowCount rows,
                         void* dst, hipStream_t st) {
    const int n_rows = rows.n;          // the grid covers the upper bound; blocks past the live count leave at once
    if (n_rows <= 0) return hipSuccess;
    const bool vec16 = (cols_bytes % 16 == 0) && ((uintptr_t)src % 16 == 0) && ((uintptr_t)dst % 16 == 0);
    const int wbytes = vec16 ? 16 : 4;
    const int words = (int)(cols_bytes / wbytes);
    int lanes = 256;
    while (lanes > 1 && lanes / 2 >= words) lanes /= 2;   // smallest power of two >= words, capped at 256
    const int rpb = 256 / lanes;
    const int grid = ceil_div(n_rows, rpb);
    if (vec16)
        gather_rows_kernel<uint4><<<grid, 256, 0, st>>>(static_cast<const uint4*>(src), idx, n_rows, rows.dev,
                                                        words, lanes, rpb, static_cast<uint4*>(dst));
    else
        gather_rows_kernel<unsigned><<<grid, 256, 0, st>>>(static_cast<const unsigned*>(src), idx,
                                                           n_rows, rows.dev, words, lanes, rpb,
                                                           static_cast<unsigned*>(dst));
    return hipGetLastError();
}

__global__ void fill_zero_kernel(uint4* p, size_t n16, unsigned char* tail, int ntail) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
    if (blockIdx.x == 0 && (int)threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
    if (bytes == 0) return hipSuccess;
    // pointers handed in by callers are at least 16-byte aligned (checked at the API)
    size_t n16 = bytes / 16;
    int ntail = (int)(bytes % 16);
    int grid = (int)((n16 + 255) / 256);
    if (grid < 1) grid = 1;
    if (grid > 4096) grid = 4096;
    fill_zero_kernel<<<grid, 256, 0, st>>>(static_cast<uint4*>(p), n16,
                                           static_cast<unsigned char*>(p) + n16 * 16, ntail);
    return hipGetLastError();
}

// dst [cols, rows] = src [rows, cols]^T through a 32x32 LDS tile
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ src, int rows, int cols,
                                                        T* __restrict__ dst) {
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = src[(int64_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) dst[(int64_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

hipError_t launch_transpose(int dtype, const void* src, int rows, int cols, void* dst, hipStream_t st) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    const dim3 grid(ceil_div(cols, 32), ceil_div(rows, 32));
    if (dtype == CF_F32)
        transpose_kernel<float><<<grid, 256, 0, st>>>((const float*)src, rows, cols, (float*)dst);
    else
        transpose_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)src, rows, cols, (bf16_t*)dst);
    return hipGetLastError();
}

}  // namespace cf
