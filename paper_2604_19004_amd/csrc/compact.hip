// Compaction (paper Section 3.2): in the estimation workflows a row's entries
// sit in a region reserved from its predicted size, so once the true sizes are
// known the rows are copied to their final, contiguous CSR positions.
#include "ocean_internal.hpp"

namespace ocean {

// One group of 2^g_log2 lanes per row.  Source of a row: the first attempt's
// region unless the row overflowed there (nnz1 < 0), then the retry's region.
template <typename V>
__global__ void __launch_bounds__(256)
k_compact(int64_t m, int g_log2, const int64_t *__restrict__ c_rp, const int32_t *__restrict__ nnz1,
          const int64_t *__restrict__ ptr1, const int32_t *__restrict__ col1, const V *__restrict__ val1,
          const int64_t *__restrict__ ptr2, const int32_t *__restrict__ col2, const V *__restrict__ val2,
          int32_t *__restrict__ c_col, V *__restrict__ c_val)
{
    const int G = 1 << g_log2;
    const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t row = gt >> g_log2;
    const int sub = (int)(gt & (G - 1));
    if (row >= m) return;
    const int64_t dst = c_rp[row];
    const int64_t n = c_rp[row + 1] - dst;
    if (n == 0) return;
    const bool first = nnz1[row] >= 0;
    const int64_t src = first ? ptr1[row] : ptr2[row];
    const int32_t *sc = first ? col1 : col2;
    const V *sv = first ? val1 : val2;
    // eight elements in flight per lane: a long row is bound by the latency of its loads otherwise
    int64_t t = sub;
    for (; t + 7 * (int64_t)G < n; t += 8 * (int64_t)G) {
        int32_t cc[8];
        V vv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { cc[i] = sc[src + t + (int64_t)i * G]; vv[i] = sv[src + t + (int64_t)i * G]; }
#pragma unroll
        for (int i = 0; i < 8; ++i) { c_col[dst + t + (int64_t)i * G] = cc[i]; c_val[dst + t + (int64_t)i * G] = vv[i]; }
    }
    // the rest four at a time, loads before stores: a short row is all "rest", and one load per lane in flight
    // left the copy of a matrix of short rows bound by latency
    for (; t < n; t += 4 * (int64_t)G) {
        int32_t cc[4];
        V vv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t u = t + (int64_t)i * G;
            cc[i] = 0; vv[i] = V();
            if (u < n) { cc[i] = sc[src + u]; vv[i] = sv[src + u]; }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t u = t + (int64_t)i * G;
            if (u < n) { c_col[dst + u] = cc[i]; c_val[dst + u] = vv[i]; }
        }
    }
}

// The same copy dealt out by entries of C instead of rows: every workgroup takes a tile of
// CF_TILE consecutive entries of C, so that the stores of the whole grid sweep C linearly and the
// loads sweep the temporary output in the same order (rows lie there in row order too), whatever
// the lengths of the rows.  This is what a power-law C needs: with a lane group per row its long
// rows turn the copy into thousands of independent streams.  The first and last row of a tile are
// found by a search over row_ptr in which all 256 threads probe at once.
constexpr int CF_THREADS = 256;
constexpr int CF_TILE = CF_THREADS * 64;

// Largest r in [0, m) with c_rp[r] <= pos (pos < c_rp[m]; rows without entries are skipped).  Uniform.
__device__ __forceinline__ int64_t row_of_entry(const int64_t *__restrict__ c_rp, int64_t m, int64_t pos)
{
    int64_t lo = 0, hi = m;   // the answer lies in [lo, hi)
    while (hi - lo > 1) {
        const int64_t step = (hi - lo + CF_THREADS - 1) / CF_THREADS;
        const int64_t idx = lo + (int64_t)threadIdx.x * step;
        const bool le = idx < hi && c_rp[idx] <= pos;
        const int cnt = __syncthreads_count(le);   // >= 1, since c_rp[lo] <= pos
        const int64_t nlo = lo + (int64_t)(cnt - 1) * step;
        hi = nlo + step < hi ? nlo + step : hi;
        lo = nlo;
    }
    return lo;
}

// Entries [first, last) of C are copied; entry e goes to c_col / c_val [e - dst_off] (dst_off = 0: C itself;
// dst_off = first: a staging buffer that starts at the range's first entry).  No __restrict__ on the
// destination and the first attempt's arrays: the in-place compaction passes the same allocation for both,
// with ranges chosen by the host so that what one launch writes lies below everything it or a later launch
// still reads.
template <typename V>
__global__ void __launch_bounds__(CF_THREADS)
k_compact_flat(int64_t m, int64_t first_entry, int64_t last_entry, int64_t dst_off, const int64_t *__restrict__ c_rp,
               const int32_t *__restrict__ nnz1, const int64_t *__restrict__ ptr1, const int32_t *col1, const V *val1,
               const int64_t *__restrict__ ptr2, const int32_t *__restrict__ col2, const V *__restrict__ val2,
               int32_t *c_col, V *c_val)
{
    const int tid = threadIdx.x;
    const int64_t nnz = last_entry;
    const int64_t base = first_entry + (int64_t)blockIdx.x * CF_TILE;
    if (base >= nnz) return;   // uniform
    const int64_t end = base + CF_TILE < nnz ? base + CF_TILE : nnz;
    c_col -= dst_off;
    c_val -= dst_off;
    const int64_t r_lo = row_of_entry(c_rp, m, base);
    const int64_t r_hi = row_of_entry(c_rp, m, end - 1);
    if (r_hi - r_lo < 64) {
        // few rows in the tile: thread t copies entries base + t, base + t + 256, ...; the row of an entry
        // only moves forward, so a thread advances over at most 64 rows in all
        int64_t row = r_lo;
        int64_t row_end = c_rp[row + 1];
        bool first = nnz1[row] >= 0;
        int64_t delta = (first ? ptr1[row] : ptr2[row]) - c_rp[row];   // position in the source minus position in C
        for (int64_t e0 = base + tid; e0 < end; e0 += 8 * CF_THREADS) {
            int32_t cc[8];
            V vv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t e = e0 + (int64_t)i * CF_THREADS;
                cc[i] = 0; vv[i] = V();
                if (e < end) {
                    while (e >= row_end) {   // (row < r_hi here: the tile ends inside row r_hi)
                        ++row;
                        row_end = c_rp[row + 1];
                        if (e < row_end) {
                            first = nnz1[row] >= 0;
                            delta = (first ? ptr1[row] : ptr2[row]) - c_rp[row];
                        }
                    }
                    const int64_t sp = e + delta;
                    cc[i] = first ? col1[sp] : col2[sp];
                    vv[i] = first ? val1[sp] : val2[sp];
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int64_t e = e0 + (int64_t)i * CF_THREADS;
                if (e < end) { c_col[e] = cc[i]; c_val[e] = vv[i]; }
            }
        }
    } else {
        // many short rows: one wave per row, the rows of the tile dealt out to the four waves
        const int lane = tid & (WAVE - 1);
        for (int64_t row = r_lo + tid / WAVE; row <= r_hi; row += CF_THREADS / WAVE) {
            const int64_t d0 = c_rp[row], d1 = c_rp[row + 1];
            const int64_t from = d0 > base ? d0 : base, to = d1 < end ? d1 : end;
            if (from >= to) continue;
            const bool first = nnz1[row] >= 0;
            const int64_t delta = (first ? ptr1[row] : ptr2[row]) - d0;
            const int32_t *sc = first ? col1 : col2;
            const V *sv = first ? val1 : val2;
            for (int64_t e = from + lane; e < to; e += WAVE) {
                c_col[e] = sc[e + delta];
                c_val[e] = sv[e + delta];
            }
        }
    }
}

hipError_t launch_compact(int64_t m, int dtype, const int64_t *c_rp, const int32_t *nnz1, const int64_t *ptr1,
                          const int32_t *col1, const void *val1, const int64_t *ptr2, const int32_t *col2,
                          const void *val2, int32_t *c_col, void *c_val, int g_log2, int64_t nnz_c, hipStream_t s)
{
    if (m == 0) return hipSuccess;
    if (nnz_c >= (int64_t)512 * m && nnz_c > 0) {   // long rows on average: deal the copy out by entries
        const int64_t tiles = (nnz_c + CF_TILE - 1) / CF_TILE;
        if (dtype == OCEAN_F64)
            hipLaunchKernelGGL(k_compact_flat<double>, dim3((unsigned)tiles), dim3(CF_THREADS), 0, s, m, (int64_t)0, nnz_c,
                               (int64_t)0, c_rp, nnz1, ptr1, col1, static_cast<const double *>(val1), ptr2, col2,
                               static_cast<const double *>(val2), c_col, static_cast<double *>(c_val));
        else
            hipLaunchKernelGGL(k_compact_flat<float>, dim3((unsigned)tiles), dim3(CF_THREADS), 0, s, m, (int64_t)0, nnz_c,
                               (int64_t)0, c_rp, nnz1, ptr1, col1, static_cast<const float *>(val1), ptr2, col2,
                               static_cast<const float *>(val2), c_col, static_cast<float *>(c_val));
        return hipGetLastError();
    }
    const int64_t threads = m << g_log2;
    const int64_t blocks = (threads + 255) / 256;
    if (dtype == OCEAN_F64)
        hipLaunchKernelGGL(k_compact<double>, dim3((unsigned)blocks), dim3(256), 0, s, m, g_log2, c_rp, nnz1, ptr1, col1,
                           static_cast<const double *>(val1), ptr2, col2, static_cast<const double *>(val2), c_col,
                           static_cast<double *>(c_val));
    else
        hipLaunchKernelGGL(k_compact<float>, dim3((unsigned)blocks), dim3(256), 0, s, m, g_log2, c_rp, nnz1, ptr1, col1,
                           static_cast<const float *>(val1), ptr2, col2, static_cast<const float *>(val2), c_col,
                           static_cast<float *>(c_val));
    return hipGetLastError();
}

// Entries [first, last) of C from their places in the two temporary outputs to dst[e - dst_off].
hipError_t launch_compact_range(int64_t m, int dtype, const int64_t *c_rp, const int32_t *nnz1, const int64_t *ptr1,
                                const int32_t *col1, const void *val1, const int64_t *ptr2, const int32_t *col2,
                                const void *val2, int32_t *dst_col, void *dst_val, int64_t first, int64_t last,
                                int64_t dst_off, hipStream_t s)
{
    if (last <= first) return hipSuccess;
    const int64_t tiles = (last - first + CF_TILE - 1) / CF_TILE;
    if (dtype == OCEAN_F64)
        hipLaunchKernelGGL(k_compact_flat<double>, dim3((unsigned)tiles), dim3(CF_THREADS), 0, s, m, first, last, dst_off, c_rp,
                           nnz1, ptr1, col1, static_cast<const double *>(val1), ptr2, col2, static_cast<const double *>(val2),
                           dst_col, static_cast<double *>(dst_val));
    else
        hipLaunchKernelGGL(k_compact_flat<float>, dim3((unsigned)tiles), dim3(CF_THREADS), 0, s, m, first, last, dst_off, c_rp,
                           nnz1, ptr1, col1, static_cast<const float *>(val1), ptr2, col2, static_cast<const float *>(val2),
                           dst_col, static_cast<float *>(dst_val));
    return hipGetLastError();
}

}  // namespace ocean
