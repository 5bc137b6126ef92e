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

__global__ __launch_bounds__(IDX_THREADS) void mask_count_kernel(const uint8_t* __restrict__ mask,
                                                                 int64_t T, int aligned,
                                                                 int32_t* __restrict__ block_count) {
    __shared__ int red[4];
    unsigned w[4];
    int64_t t0 = (int64_t)blockIdx.x * IDX_CHUNK + (int64_t)threadIdx.x * IDX_PER_THREAD;
    load_flags(mask, t0, T, aligned != 0, w);
    int total = block_sum_256(count_flags(w), red);
    if (threadIdx.x == 0) block_count[blockIdx.x] = total;
}

// Exclusive prefix sum of the per-block counts, in place: one block, each thread owns a
// contiguous run of the array.
__global__ __launch_bounds__(1024) void block_scan_kernel(int32_t* __restrict__ block_count, int nblk) {
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int per = (nblk + 1023) / 1024;
    const int lo = min(tid * per, nblk), hi = min(lo + per, nblk);
    int s = 0;
    for (int i = lo; i < hi; ++i) s += block_count[i];
    part[tid] = s;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {        // Hillis-Steele inclusive scan of the 1024 run totals
        const int v = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    int run = part[tid] - s;                    // exclusive
    for (int i = lo; i < hi; ++i) {
        const int c = block_count[i];
        block_count[i] = run;
        run += c;
    }
}

// block_count == nullptr: every block counts the mask bytes before its chunk itself
// (only used for a handful of blocks); otherwise block_count[b] holds the number of kept
// tokens before chunk b.
__global__ __launch_bounds__(IDX_THREADS) void mask_scatter_kernel(
    const uint8_t* __restrict__ mask, int64_t T, int S, int B, int aligned,
    const int32_t* __restrict__ block_count, int32_t* __restrict__ idx,
    int32_t* __restrict__ cu_kept, int32_t* __restrict__ n_kept_dev) {
    __shared__ int red[4];
    __shared__ int wave_tot[4];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;

    int base;
    if (block_count != nullptr) {
        base = block_count[blockIdx.x];
    } else {
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

size_t index_ws_bytes(int64_t n_tokens) {
    int64_t nblk = (n_tokens + IDX_CHUNK - 1) / IDX_CHUNK;
    if (nblk < 1) nblk = 1;
    return align_up((size_t)nblk * sizeof(int32_t), 256);
}

hipError_t launch_keep_index(const uint8_t* mask, int B, int S, int32_t* idx, int32_t* cu_kept,
                             int32_t* n_kept_dev, void* ws, hipStream_t st) {
    const int64_t T = (int64_t)B * S;
    const int nblk = ceil_div(T, IDX_CHUNK);
    const int aligned = ((uintptr_t)mask % 16 == 0) ? 1 : 0;
    if (nblk <= IDX_SELF_COUNT_MAX_BLOCKS) {
        mask_scatter_kernel<<<nblk, IDX_THREADS, 0, st>>>(mask, T, S, B, aligned, nullptr, idx,
                                                          cu_kept, n_kept_dev);
    } else {
        int32_t* block_count = static_cast<int32_t*>(ws);
        mask_count_kernel<<<nblk, IDX_THREADS, 0, st>>>(mask, T, aligned, block_count);
        block_scan_kernel<<<1, 1024, 0, st>>>(block_count, nblk);
        mask_scatter_kernel<<<nblk, IDX_THREADS, 0, st>>>(mask, T, S, B, aligned, block_count, idx,
                                                          cu_kept, n_kept_dev);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// The same index build for callers that cannot allocate or hand in a workspace: the per-block
// counts live in a file-scope device array.  Every GPU holds its own copy of the array at its own
// address; host code never uses the array's name as a pointer but looks its address up once per
// device (with that device current) and passes that pointer to the kernels.  The kernels write
// every entry they later read (block b's count, b < number of blocks), so nothing has to be
// cleared between calls; calls that overlap on one GPU share the array and race.
// ---------------------------------------------------------------------------
static __device__ __align__(256) int32_t scratch[IDX_STATIC_MAX_TOKENS / IDX_CHUNK];

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
