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
    for (; t < n; t += G) {
        c_col[dst + t] = sc[src + t];
        c_val[dst + t] = sv[src + t];
    }
}

hipError_t launch_compact(int64_t m, int dtype, const int64_t *c_rp, const int32_t *nnz1, const int64_t *ptr1,
                          const int32_t *col1, const void *val1, const int64_t *ptr2, const int32_t *col2,
                          const void *val2, int32_t *c_col, void *c_val, int g_log2, hipStream_t s)
{
    if (m == 0) return hipSuccess;
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

}  // namespace ocean
