// Order of the rows inside the launch of the heavy-row kernel.  Its persistent
// workgroups take rows one by one from the end of the list; a row of a
// power-law matrix can hold a hundred times the work of the median row of its
// bin, and one that is handed out late keeps a single CU busy long after all
// others have finished.  Handing out the longest rows first needs no exact
// sort: rows are ordered by a coarse key of their product count (its binary
// exponent and the three bits below the leading one, i.e. classes 12 % wide)
// with one counting pass - count per class, prefix sum, scatter.  The order
// inside a class is whatever the atomics give; it has no effect on the result.
#include "ocean_internal.hpp"

namespace ocean {

namespace {
constexpr int OB_CLASSES = 512;   // 64 exponents x 8
constexpr int OB_THREADS = 256;
constexpr int OB_ITEMS = 8;       // rows per thread of the scatter
constexpr size_t SORT_ALIGN = 256;
inline size_t sort_up(size_t b) { return (b + SORT_ALIGN - 1) / SORT_ALIGN * SORT_ALIGN; }

__device__ __forceinline__ int product_class(int64_t p)
{
    if (p <= 0) return 0;
    const int e = 63 - __clzll((long long)p);
    const int m = e >= 3 ? (int)((p >> (e - 3)) & 7) : (int)((p << (3 - e)) & 7);
    return e * 8 + m;   // < 512, monotone in p
}

__global__ void __launch_bounds__(OB_THREADS)
k_order_count(const int64_t *__restrict__ prod, const int32_t *__restrict__ rows, int64_t count, unsigned int *hist)
{
    __shared__ unsigned int s_hist[OB_CLASSES];
    for (int j = threadIdx.x; j < OB_CLASSES; j += OB_THREADS) s_hist[j] = 0u;
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * OB_THREADS + threadIdx.x; i < count; i += (int64_t)gridDim.x * OB_THREADS)
        atomicAdd(&s_hist[product_class(prod[rows[i]])], 1u);
    __syncthreads();
    for (int j = threadIdx.x; j < OB_CLASSES; j += OB_THREADS)
        if (s_hist[j]) atomicAdd(&hist[j], s_hist[j]);
}

// counts -> first position of every class (exclusive prefix sum), in place; one workgroup of OB_CLASSES threads
__global__ void __launch_bounds__(OB_CLASSES)
k_order_scan(unsigned int *hist)
{
    __shared__ unsigned int s_part[OB_CLASSES / WAVE];
    const unsigned int v = hist[threadIdx.x];
    const unsigned int inc = wave_inclusive_scan_u32(v);
    if (lane_id() == WAVE - 1) s_part[threadIdx.x / WAVE] = inc;
    __syncthreads();
    uint32_t total;
    const uint32_t before = waves_before_u32<OB_CLASSES / WAVE>(s_part, (int)threadIdx.x / WAVE, total);
    hist[threadIdx.x] = before + inc - v;
}

// A workgroup ranks its tile of rows per class in LDS, claims one range per class, and writes its rows there.
__global__ void __launch_bounds__(OB_THREADS)
k_order_scatter(const int64_t *__restrict__ prod, const int32_t *__restrict__ rows, int64_t count,
                unsigned int *cursor, int32_t *__restrict__ out)
{
    __shared__ unsigned int s_cnt[OB_CLASSES];
    __shared__ unsigned int s_base[OB_CLASSES];
    for (int j = threadIdx.x; j < OB_CLASSES; j += OB_THREADS) s_cnt[j] = 0u;
    __syncthreads();
    const int64_t tile = (int64_t)blockIdx.x * OB_THREADS * OB_ITEMS;
    int32_t row[OB_ITEMS];
    int cls[OB_ITEMS];
    unsigned int rank[OB_ITEMS];
#pragma unroll
    for (int q = 0; q < OB_ITEMS; ++q) {
        const int64_t i = tile + (int64_t)q * OB_THREADS + threadIdx.x;
        cls[q] = -1; row[q] = 0; rank[q] = 0;
        if (i < count) {
            row[q] = rows[i];
            cls[q] = product_class(prod[row[q]]);
            rank[q] = atomicAdd(&s_cnt[cls[q]], 1u);
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < OB_CLASSES; j += OB_THREADS)
        s_base[j] = s_cnt[j] ? atomicAdd(&cursor[j], s_cnt[j]) : 0u;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < OB_ITEMS; ++q)
        if (cls[q] >= 0) out[s_base[cls[q]] + rank[q]] = row[q];
}
}  // namespace

// ---- a copy of B with every row's entries in column order -------------------------------------------
// Needed when B's rows come unsorted and so much work sits in heavy rows that the kernels which accumulate
// in global memory would be bound by atomic throughput (the case Section 5.4 reports for the enhanced hash
// accumulator): the column-window kernel needs sorted rows.  One workgroup per row: column ids and the
// entries' positions go to LDS, a bitonic network orders them, the values follow their positions (indirect
// sort, Section 4.2).  Rows longer than SB_MAX are copied unsorted: flags |= 16 and the caller keeps B as it is.
namespace {
constexpr int SB_THREADS = 256;
constexpr int SB_MAX = 4096;

template <typename V>
__global__ void __launch_bounds__(SB_THREADS)
k_sort_b_rows(const int64_t *__restrict__ rp, const int32_t *__restrict__ col, const V *__restrict__ val, int64_t rows,
              int32_t *__restrict__ col_out, V *__restrict__ val_out, int32_t *flags)
{
    __shared__ int32_t s_key[SB_MAX];
    __shared__ uint16_t s_pos[SB_MAX];
    for (int64_t row = blockIdx.x; row < rows; row += gridDim.x) {
        const int64_t p0 = rp[row];
        const int64_t full = rp[row + 1] - p0;
        const int len = (int)(full > SB_MAX + 1 ? SB_MAX + 1 : full);
        if (len > SB_MAX) {   // uniform: copied as it is, so that the copy stays a valid matrix (its column ids are in range)
            if (threadIdx.x == 0) atomicOr(flags, 16);
            for (int64_t i = threadIdx.x; i < full; i += SB_THREADS) { col_out[p0 + i] = col[p0 + i]; val_out[p0 + i] = val[p0 + i]; }
            continue;
        }
        if (len <= 1) {
            if (len == 1 && threadIdx.x == 0) { col_out[p0] = col[p0]; val_out[p0] = val[p0]; }
            continue;
        }
        int n = 2;
        while (n < len) n <<= 1;
        for (int i = threadIdx.x; i < n; i += SB_THREADS) {
            s_key[i] = i < len ? col[p0 + i] : SORT_PAD;
            s_pos[i] = (uint16_t)i;
        }
        __syncthreads();
        for (int k = 2; k <= n; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int i = threadIdx.x; i < (n >> 1); i += SB_THREADS) {
                    const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                    const int hi = lo | j;
                    const int32_t x = s_key[lo], y = s_key[hi];
                    if ((x > y) == ((lo & k) == 0)) {
                        s_key[lo] = y; s_key[hi] = x;
                        const uint16_t t = s_pos[lo]; s_pos[lo] = s_pos[hi]; s_pos[hi] = t;
                    }
                }
                __syncthreads();
            }
        }
        for (int i = threadIdx.x; i < len; i += SB_THREADS) {
            col_out[p0 + i] = s_key[i];
            val_out[p0 + i] = val[p0 + s_pos[i]];
        }
        __syncthreads();   // the arrays are rewritten for the next row
    }
}
}  // namespace

hipError_t launch_sort_b_rows(const Csr &B, int dtype, int32_t *col_out, void *val_out, int32_t *flags, hipStream_t s)
{
    if (B.rows == 0 || B.nnz == 0) return hipSuccess;
    const int64_t blocks = B.rows < 65536 ? B.rows : 65536;
    if (dtype == OCEAN_F64)
        hipLaunchKernelGGL(k_sort_b_rows<double>, dim3((unsigned)blocks), dim3(SB_THREADS), 0, s, B.rp, B.col,
                           static_cast<const double *>(B.val), B.rows, col_out, static_cast<double *>(val_out), flags);
    else
        hipLaunchKernelGGL(k_sort_b_rows<float>, dim3((unsigned)blocks), dim3(SB_THREADS), 0, s, B.rp, B.col,
                           static_cast<const float *>(B.val), B.rows, col_out, static_cast<float *>(val_out), flags);
    return hipGetLastError();
}

size_t sort_rows_scratch_bytes(int64_t count)
{
    if (count <= 1 || count > 0x7fffffffLL) return 0;
    return sort_up((size_t)OB_CLASSES * sizeof(unsigned int)) + sort_up((size_t)count * 4);
}

// rows[0..count) reordered in place by ascending class of their product counts.  scratch:
// sort_rows_scratch_bytes(count) bytes.
hipError_t launch_sort_rows_by_products(const int64_t *prod, int32_t *rows, int64_t count, void *scratch, hipStream_t s)
{
    if (count <= 1 || count > 0x7fffffffLL) return hipSuccess;
    char *base = static_cast<char *>(scratch);
    unsigned int *hist = reinterpret_cast<unsigned int *>(base);
    int32_t *rows_out = reinterpret_cast<int32_t *>(base + sort_up((size_t)OB_CLASSES * sizeof(unsigned int)));
    hipError_t e = hipMemsetAsync(hist, 0, (size_t)OB_CLASSES * sizeof(unsigned int), s);
    if (e != hipSuccess) return e;
    int64_t blocks = (count + OB_THREADS * OB_ITEMS - 1) / (OB_THREADS * OB_ITEMS);
    const int64_t count_blocks = blocks < 512 ? blocks : 512;
    hipLaunchKernelGGL(k_order_count, dim3((unsigned)count_blocks), dim3(OB_THREADS), 0, s, prod, rows, count, hist);
    hipLaunchKernelGGL(k_order_scan, dim3(1), dim3(OB_CLASSES), 0, s, hist);
    hipLaunchKernelGGL(k_order_scatter, dim3((unsigned)blocks), dim3(OB_THREADS), 0, s, prod, rows, count, hist, rows_out);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return hipMemcpyAsync(rows, rows_out, (size_t)count * 4, hipMemcpyDeviceToDevice, s);
}

}  // namespace ocean
