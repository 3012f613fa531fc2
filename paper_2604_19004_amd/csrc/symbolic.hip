// Exact symbolic pass (paper Section 2.3): the number of distinct output
// columns of every row, by Gustavson's traversal with values dropped.  This is
// the size prediction of the two-pass workflow that the estimation workflow
// is measured against, so it gets the same care: key-only LDS hash tables
// binned by the product-count upper bound, and for rows whose bound exceeds
// any key table an LDS bitmap over windows of 2^20 columns (one fire-and-forget
// LDS OR per product, a popcount at the end).
#include "ocean_internal.hpp"
#include "traverse.hpp"

namespace ocean {

// 1: key was new, 0: already present, -1: table full
template <int BITS>
__device__ __forceinline__ int lds_insert_new(int32_t *keys, int32_t key)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    uint32_t h = table_hash(key, BITS);
    for (uint32_t probe = 0; probe <= MASK; ++probe) {
        const int32_t cur = __hip_atomic_load(&keys[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (cur == key) return 0;
        if (cur == EMPTY_KEY) {
            const int32_t old = atomicCAS(&keys[h], EMPTY_KEY, key);
            if (old == EMPTY_KEY) return 1;
            if (old == key) return 0;
        }
        h = (h + 1u) & MASK;
    }
    return -1;
}

using NoVal = unsigned char;   // the symbolic pass carries no values

// ---------------------------------------------------------- group kernel
template <int G, int BITS>
__global__ void __launch_bounds__(256)
k_symbolic_group(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
                 const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col,
                 const int32_t *__restrict__ rows, int64_t count, int gb_log2, int32_t *__restrict__ nnz_out)
{
    constexpr int SLOTS = 1 << BITS;
    constexpr int R = 256 / G;
    __shared__ int32_t s_keys[R * SLOTS];
    const int rl = threadIdx.x / G;
    const int sub = threadIdx.x % G;
    int32_t *keys = s_keys + rl * SLOTS;
    const int gb = 1 << gb_log2;
    const int sub_b = sub & (gb - 1);
    const int part = sub >> gb_log2;
    const int parts = G >> gb_log2;
    const int64_t r = (int64_t)blockIdx.x * R + rl;
    const bool live = r < count;
    const int64_t row = live ? rows[r] : 0;
    for (int s = sub; s < SLOTS; s += G) keys[s] = EMPTY_KEY;
    wave_sync();
    int fresh = 0;
    if (live) {
        const int64_t e1 = a_rp[row + 1];
        for (int64_t e = a_rp[row] + part; e < e1; e += parts) {
            const int64_t k = a_col[e];
            const int64_t p1 = b_rp[k + 1];
            for (int64_t p = b_rp[k] + sub_b; p < p1; p += gb) fresh += (lds_insert_new<BITS>(keys, b_col[p]) == 1);
        }
    }
    fresh = group_reduce_sum(fresh, G);
    if (live && sub == 0) nnz_out[row] = fresh;
}

// ----------------------------------------------------------- wave kernel
__global__ void __launch_bounds__(256)
k_symbolic_wave(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
                const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col,
                const int32_t *__restrict__ rows, int64_t count, int32_t *__restrict__ nnz_out)
{
    constexpr int BITS = 8;
    constexpr int SLOTS = 1 << BITS;
    __shared__ int32_t s_keys[4 * SLOTS];
    __shared__ WaveQueue<NoVal> s_q[4];
    const int rl = threadIdx.x / WAVE;
    const int sub = lane_id();
    int32_t *keys = s_keys + rl * SLOTS;
    const int64_t r = (int64_t)blockIdx.x * 4 + rl;
    if (r >= count) return;   // no workgroup barrier below
    const int64_t row = rows[r];
    for (int s = sub; s < SLOTS; s += WAVE) keys[s] = EMPTY_KEY;
    wave_sync();
    int fresh = 0;
    wave_traverse<false>(a_col, (const NoVal *)nullptr, a_rp[row], a_rp[row + 1],
                         [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                         b_col, (const NoVal *)nullptr, s_q[rl],
                         [&](int32_t j, NoVal) { fresh += (lds_insert_new<BITS>(keys, j) == 1); });
    fresh = group_reduce_sum(fresh, WAVE);
    if (sub == 0) nnz_out[row] = fresh;
}

// ------------------------------------------------------ workgroup kernel
template <int BITS, int THREADS>
__global__ void __launch_bounds__(THREADS)
k_symbolic_wg(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
              const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col,
              const int32_t *__restrict__ rows, int64_t count, int32_t *__restrict__ nnz_out)
{
    constexpr int SLOTS = 1 << BITS;
    __shared__ int32_t s_keys[SLOTS];
    __shared__ TravQueue<NoVal, THREADS> s_q;
    __shared__ int s_count;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (r >= count) return;
    const int64_t row = rows[r];
    for (int s = tid; s < SLOTS; s += THREADS) s_keys[s] = EMPTY_KEY;
    if (tid == 0) { s_count = 0; s_q.n = 0; s_q.n_huge = 0; }
    __syncthreads();
    int fresh = 0;
    TravState ts;
    wg_traverse<THREADS, false>(a_col, (const NoVal *)nullptr, a_rp[row], a_rp[row + 1],
                                [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                b_col, (const NoVal *)nullptr, s_q, ts,
                                [&](int32_t j, NoVal) { fresh += (lds_insert_new<BITS>(s_keys, j) == 1); });
    fresh = group_reduce_sum(fresh, WAVE);
    if (lane_id() == 0 && fresh) atomicAdd(&s_count, fresh);
    __syncthreads();
    if (tid == 0) nnz_out[row] = s_count;
}

// --------------------------------------------------------- bitmap kernel
constexpr int BM_THREADS = 1024;
constexpr int BM_WIN = 1 << 20;          // columns per window
constexpr int BM_WORDS = BM_WIN / 32;    // 32768 words = 128 KB

__global__ void __launch_bounds__(BM_THREADS)
k_symbolic_bitmap(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
                  const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col,
                  const int32_t *__restrict__ rows, int64_t count, int64_t n_cols,
                  unsigned long long *queue, int32_t *__restrict__ nnz_out)
{
    __shared__ uint32_t s_bm[BM_WORDS];
    __shared__ TravQueue<NoVal, BM_THREADS> s_q;
    __shared__ int s_count;
    __shared__ long long s_row;
    const int tid = threadIdx.x;
    for (int s = tid; s < BM_WORDS; s += BM_THREADS) s_bm[s] = 0u;
    for (;;) {
        if (tid == 0) { s_row = (long long)atomicAdd(queue, 1ull); s_count = 0; s_q.n = 0; s_q.n_huge = 0; }
        __syncthreads();
        const int64_t r = s_row;
        if (r >= count) break;   // uniform exit
        const int64_t row = rows[r];
        const int64_t e0 = a_rp[row], e1 = a_rp[row + 1];
        TravState ts;   // reset with the queue counters above; runs on over the windows of this row
        for (int64_t w0 = 0; w0 < n_cols; w0 += BM_WIN) {
            wg_traverse<BM_THREADS, false>(a_col, (const NoVal *)nullptr, e0, e1,
                                           [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                           b_col, (const NoVal *)nullptr, s_q, ts, [&](int32_t j, NoVal) {
                                               const int64_t d = (int64_t)j - w0;
                                               if (d >= 0 && d < BM_WIN) atomicOr(&s_bm[d >> 5], 1u << (d & 31));
                                           });
            __syncthreads();
            int c = 0;
            for (int s = tid; s < BM_WORDS; s += BM_THREADS) { c += __popc(s_bm[s]); s_bm[s] = 0u; }
            c = group_reduce_sum(c, WAVE);
            if (lane_id() == 0 && c) atomicAdd(&s_count, c);
            __syncthreads();
        }
        if (tid == 0) nnz_out[row] = s_count;
        __syncthreads();
    }
}

// -------------------------------------------------------------- dispatch
hipError_t launch_symbolic_bin(const Csr &A, const Csr &B, const SymLaunch &l, int gb_log2, int32_t *nnz_out,
                               int n_wg, unsigned long long *queue, hipStream_t s)
{
    if (l.count <= 0) return hipSuccess;
#define OCEAN_SYM_WG(BITS, THREADS)                                                                               \
    hipLaunchKernelGGL((k_symbolic_wg<BITS, THREADS>), dim3((unsigned)l.count), dim3(THREADS), 0, s, A.rp, A.col,   \
                       B.rp, B.col, l.rows, l.count, nnz_out)
    switch (l.bin) {
    case SB_G16:
        hipLaunchKernelGGL((k_symbolic_group<16, 6>), dim3((unsigned)((l.count + 15) / 16)), dim3(256), 0, s, A.rp, A.col,
                           B.rp, B.col, l.rows, l.count, gb_log2 < 4 ? gb_log2 : 4, nnz_out);
        break;
    case SB_W64:
        hipLaunchKernelGGL(k_symbolic_wave, dim3((unsigned)((l.count + 3) / 4)), dim3(256), 0, s, A.rp, A.col, B.rp, B.col,
                           l.rows, l.count, nnz_out);
        break;
    case SB_S1K: OCEAN_SYM_WG(10, 256); break;
    case SB_S4K: OCEAN_SYM_WG(12, 512); break;
    case SB_S16K: OCEAN_SYM_WG(14, 1024); break;
    case SB_S32K: OCEAN_SYM_WG(15, 1024); break;
    case SB_BITMAP:
        hipLaunchKernelGGL(k_symbolic_bitmap, dim3((unsigned)n_wg), dim3(BM_THREADS), 0, s, A.rp, A.col, B.rp, B.col,
                           l.rows, l.count, B.cols, queue, nnz_out);
        break;
    default: return hipErrorInvalidValue;
    }
#undef OCEAN_SYM_WG
    return hipGetLastError();
}

}  // namespace ocean
