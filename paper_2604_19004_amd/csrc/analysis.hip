// Analysis step and HyperLogLog size prediction (paper Sections 2.4, 3.1, 3.2).
//
//   k_validate        input check (row offsets ascending, column ids in range)
//   k_row_products    prod[i] = sum_{k in A_i} nnz(B_k); P and the largest row; longest B row per A row
//   k_hll_sketch      construct: one m-register sketch per row of B, registers live in LDS per lane group
//   k_hll_merge       merge along each row of A (byte-wise max of 8 registers per lane) + estimate
//   k_sample_reduce   sums over the sampled rows for the sampled compression ratio
//
// All kernels are HBM/L2-bound gathers; rows are mapped to groups of G lanes
// (G a power of two <= 64 chosen from the average row length) so that short
// rows do not leave most of a 64-wide wave idle.
#include "ocean_internal.hpp"

namespace ocean {

constexpr int TPB = 256;

static inline int ilog2_ceil(double x, int lo, int hi)
{
    int l = lo;
    while (l < hi && (double)(1 << l) < x) ++l;
    return l;
}

// ---------------------------------------------------------------- validate
// near_pairs (may be null): a measure of how clustered the columns of the matrix are, taken on a sample - every
// 16th workgroup adds the number of entries it looked at to near_pairs[0] and the number of those whose
// successor's column id is 1 .. 4 larger to near_pairs[1] (pairs across a row boundary count too; they are few).
// One pair of atomics per sampling workgroup: same-address atomics serialise at about 12 ns each.
__global__ void k_validate(const int64_t *rp, const int32_t *col, int64_t rows, int64_t cols, int64_t nnz,
                           int32_t *flags, int bit, unsigned long long *near_pairs)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    const bool sampling = near_pairs != nullptr && (blockIdx.x & 15u) == 0u;   // uniform
    unsigned int near = 0, seen = 0;
    for (int64_t i = t0; i < rows; i += stride) {
        int64_t a = rp[i], b = rp[i + 1];
        bad |= (b < a) | (a < 0) | (b > nnz);
    }
    if (t0 == 0) bad |= (rp[0] != 0) | (rp[rows] != nnz);
    for (int64_t e = t0; e < nnz; e += stride) {
        int32_t c = col[e];
        bad |= ((uint32_t)c >= (uint64_t)cols);
        if (sampling && e + 1 < nnz) { near += (uint32_t)(col[e + 1] - c - 1) < 4u; ++seen; }
    }
    if (__ballot(bad) != 0 && lane_id() == 0) atomicOr(flags, bit);
    if (sampling) {
        __shared__ unsigned int s_near, s_seen;
        if (threadIdx.x == 0) { s_near = 0u; s_seen = 0u; }
        __syncthreads();
        const unsigned int wave_near = wave_sum_u32(near), wave_seen = wave_sum_u32(seen);
        if (lane_id() == 0) { atomicAdd(&s_near, wave_near); atomicAdd(&s_seen, wave_seen); }
        __syncthreads();
        if (threadIdx.x == 0 && s_seen) {
            atomicAdd(&near_pairs[0], (unsigned long long)s_seen);
            atomicAdd(&near_pairs[1], (unsigned long long)s_near);
        }
    }
}

// b_near_pairs: two zeroed device counters that receive the clustering measure of B's columns (see k_validate).
hipError_t launch_validate(const Csr &A, const Csr &B, int32_t *flags, unsigned long long *b_near_pairs, hipStream_t s)
{
    auto go = [&](const Csr &M, int bit, unsigned long long *near) {
        int64_t work = M.nnz > M.rows ? M.nnz : M.rows;
        int blocks = (int)((work + TPB * 4 - 1) / (TPB * 4));
        if (blocks < 1) blocks = 1;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(k_validate, dim3(blocks), dim3(TPB), 0, s, M.rp, M.col, M.rows, M.cols, M.nnz, flags, bit, near);
    };
    const bool same = B.rp == A.rp && B.col == A.col && B.rows == A.rows && B.cols == A.cols;
    go(A, 1, same ? b_near_pairs : nullptr);
    if (!same) go(B, 2, b_near_pairs);
    return hipGetLastError();
}

// ------------------------------------------------------------ row products
// One group of 2^g_log2 lanes per row, a fixed number of workgroups striding
// over the rows: the totals cost one atomic per workgroup, not one per row tile
// (same-address atomics from all XCDs serialise in the memory fabric).  A row
// far longer than the average would keep its few lanes busy for a long time,
// and on power-law inputs such rows cluster (their indices share bit patterns,
// so whole workgroups would get nothing else): they are put on a list and a
// second kernel gives each of them a workgroup of its own.
// Totals of the row-products pass.  Same-address atomics from all over the chip serialise in the L2 at about 12
// ns each, and there is one set per workgroup: they are spread over ROW_TOTAL_SLOTS slots of 128 bytes (one
// cache line each) by workgroup index and added up by whoever reads them (sum_row_totals on the host).
// slot[0] += products, slot[1] = max(products of a row), slot[2] += products of the rows whose product count
// exceeds heavy_from (the rows that outgrow the LDS hash tables).
__device__ __forceinline__ void block_totals(long long tsum, long long tmax, long long theavy, long long *s_sum,
                                             long long *s_max, long long *s_heavy, unsigned long long *totals)
{
    const long long wsum = group_reduce_sum(tsum, WAVE);
    const long long wmax = group_reduce_max(tmax, WAVE);
    const long long wheavy = group_reduce_sum(theavy, WAVE);
    const int w = threadIdx.x / WAVE;
    if (lane_id() == 0) { s_sum[w] = wsum; s_max[w] = wmax; s_heavy[w] = wheavy; }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long bs = 0, bm = 0, bh = 0;
        for (int i = 0; i < TPB / WAVE; ++i) { bs += s_sum[i]; bm = s_max[i] > bm ? s_max[i] : bm; bh += s_heavy[i]; }
        unsigned long long *slot = totals + (size_t)(blockIdx.x % ROW_TOTAL_SLOTS) * ROW_TOTAL_STRIDE;
        if (bs) atomicAdd(&slot[0], (unsigned long long)bs);
        if (bm) atomicMax(&slot[1], (unsigned long long)bm);
        if (bh) atomicAdd(&slot[2], (unsigned long long)bh);
    }
}

__global__ void __launch_bounds__(TPB)
k_row_products(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, int64_t m, int64_t a_nnz,
               const int64_t *__restrict__ b_rp, int64_t b_rows, int g_log2, int64_t *__restrict__ prod,
               int32_t *__restrict__ maxb, unsigned long long *totals, int32_t *flags,
               int32_t *__restrict__ long_rows, unsigned long long *long_count, int64_t heavy_from)
{
    __shared__ long long s_sum[TPB / WAVE];
    __shared__ long long s_max[TPB / WAVE];
    __shared__ long long s_heavy[TPB / WAVE];
    const int G = 1 << g_log2;
    const int R = TPB >> g_log2;
    const int rl = threadIdx.x >> g_log2;
    const int sub = threadIdx.x & (G - 1);
    const int64_t long_len = (int64_t)G * 16;
    long long tsum = 0, tmax = 0, theavy = 0;
    bool bad = false, bad_rp = false;
    for (int64_t base = (int64_t)blockIdx.x * R; base < m; base += (int64_t)gridDim.x * R) {
        const int64_t row = base + rl;
        long long p = 0, mx = 0;
        bool mine = row < m;
        if (mine) {
            // offsets outside [0, nnz] or descending are reported and never used as they stand: this kernel
            // runs before the host has seen the verdict of the input check
            int64_t e0 = a_rp[row], e1 = a_rp[row + 1];
            if (e0 < 0 || e1 < e0 || e1 > a_nnz) { bad_rp = true; e0 = 0; e1 = 0; }
            if (long_rows != nullptr && e1 - e0 > long_len) {   // uniform for the group
                if (sub == 0) long_rows[atomicAdd(long_count, 1ull)] = (int32_t)row;
                mine = false;
            }
            if (mine) {
                // four independent chains (entry -> row offsets of B) in flight per lane; reads are
                // unconditional (index clamped) so that they are issued together
                for (int64_t e = e0 + sub; e < e1; e += 4 * G) {
                    int32_t k[4];
                    bool ok[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int64_t idx = e + (int64_t)i * G;
                        ok[i] = idx < e1;
                        k[i] = a_col[ok[i] ? idx : e];
                        if ((uint32_t)k[i] >= (uint64_t)b_rows) { bad = true; k[i] = 0; ok[i] = false; }
                    }
                    long long len[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) len[i] = b_rows > 0 ? b_rp[k[i] + 1] - b_rp[k[i]] : 0;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (ok[i]) {
                            p += len[i];
                            mx = len[i] > mx ? len[i] : mx;
                        }
                    }
                }
            }
        }
        p = group_reduce_sum(p, G);
        mx = group_reduce_max(mx, G);
        if (mine && sub == 0) {
            prod[row] = p;
            maxb[row] = (int32_t)(mx > 0x7fffffffLL ? 0x7fffffffLL : mx);
            tsum += p;
            tmax = p > tmax ? p : tmax;
            theavy += p > heavy_from ? p : 0;
        }
    }
    block_totals(tsum, tmax, theavy, s_sum, s_max, s_heavy, totals);
    if (__ballot(bad) != 0 && lane_id() == 0) atomicOr(flags, 4);
    if (__ballot(bad_rp) != 0 && lane_id() == 0) atomicOr(flags, 1);
}

// The listed long rows: one workgroup per row at a time.
__global__ void __launch_bounds__(TPB)
k_row_products_long(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
                    const int64_t *__restrict__ b_rp, int64_t b_rows, int64_t *__restrict__ prod,
                    int32_t *__restrict__ maxb, unsigned long long *totals, int32_t *flags,
                    const int32_t *__restrict__ long_rows, const unsigned long long *long_count, int64_t heavy_from)
{
    __shared__ long long s_sum[TPB / WAVE];
    __shared__ long long s_max[TPB / WAVE];
    __shared__ long long s_heavy[TPB / WAVE];
    const int64_t n = (int64_t)*long_count;
    const int w = threadIdx.x / WAVE;
    long long tsum = 0, tmax = 0, theavy = 0;
    bool bad = false;
    for (int64_t i = blockIdx.x; i < n; i += gridDim.x) {
        const int64_t row = long_rows[i];
        const int64_t e0 = a_rp[row], e1 = a_rp[row + 1];   // (only rows with valid offsets are listed)
        long long p = 0, mx = 0;
        for (int64_t e = e0 + threadIdx.x; e < e1; e += 4 * TPB) {
            int32_t k[4];
            bool ok[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t idx = e + (int64_t)j * TPB;
                ok[j] = idx < e1;
                k[j] = a_col[ok[j] ? idx : e];
                if ((uint32_t)k[j] >= (uint64_t)b_rows) { bad = true; k[j] = 0; ok[j] = false; }
            }
            long long len[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) len[j] = b_rows > 0 ? b_rp[k[j] + 1] - b_rp[k[j]] : 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (ok[j]) {
                    p += len[j];
                    mx = len[j] > mx ? len[j] : mx;
                }
            }
        }
        const long long wsum = group_reduce_sum(p, WAVE);
        const long long wmax = group_reduce_max(mx, WAVE);
        if (lane_id() == 0) { s_sum[w] = wsum; s_max[w] = wmax; }
        __syncthreads();
        if (threadIdx.x == 0) {
            long long rp = 0, rm = 0;
            for (int j = 0; j < TPB / WAVE; ++j) { rp += s_sum[j]; rm = s_max[j] > rm ? s_max[j] : rm; }
            prod[row] = rp;
            maxb[row] = (int32_t)(rm > 0x7fffffffLL ? 0x7fffffffLL : rm);
            tsum += rp;
            tmax = rp > tmax ? rp : tmax;
            theavy += rp > heavy_from ? rp : 0;
        }
        __syncthreads();
    }
    block_totals(tsum, tmax, theavy, s_sum, s_max, s_heavy, totals);
    if (__ballot(bad) != 0 && lane_id() == 0) atomicOr(flags, 4);
}

// long_rows: scratch for A.rows row ids, long_count: a zeroed device counter; both may be null
// (then every row is handled by its lane group).
hipError_t launch_row_products(const Csr &A, const int64_t *b_rp, int64_t b_rows, int64_t *prod, int32_t *maxb,
                               unsigned long long *totals, int32_t *flags, int32_t *long_rows,
                               unsigned long long *long_count, hipStream_t s)
{
    const int64_t heavy_from = kNumericSlots[NB_S4K];   // beyond the largest LDS hash table that sorted inputs use
    if (A.rows == 0) return hipSuccess;
    const double avg = A.rows ? (double)A.nnz / (double)A.rows : 0.0;
    const int g_log2 = ilog2_ceil(avg / 4.0, 1, 6);   // (a lane keeps four entries in flight)
    const int R = TPB >> g_log2;
    int64_t blocks = (A.rows + R - 1) / R;
    if (blocks > 2048) blocks = 2048;
    if (long_count == nullptr) long_rows = nullptr;
    hipLaunchKernelGGL(k_row_products, dim3((unsigned)blocks), dim3(TPB), 0, s, A.rp, A.col, A.rows, A.nnz, b_rp,
                       b_rows, g_log2, prod, maxb, totals, flags, long_rows, long_count, heavy_from);
    if (long_rows != nullptr)
        hipLaunchKernelGGL(k_row_products_long, dim3(2048), dim3(TPB), 0, s, A.rp, A.col, b_rp, b_rows, prod, maxb,
                           totals, flags, long_rows, long_count, heavy_from);
    return hipGetLastError();
}

// Totals of a finished row-products pass, handed to a caller-owned device array: {P, largest row, flags}.
__global__ void k_publish_totals(const unsigned long long *totals, const int32_t *flags, int64_t *out)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        unsigned long long sum = 0, mx = 0;
        for (int i = 0; i < ROW_TOTAL_SLOTS; ++i) {
            sum += totals[(size_t)i * ROW_TOTAL_STRIDE];
            const unsigned long long v = totals[(size_t)i * ROW_TOTAL_STRIDE + 1];
            mx = v > mx ? v : mx;
        }
        out[0] = (int64_t)sum;
        out[1] = (int64_t)mx;
        out[2] = (int64_t)*flags;
    }
}

hipError_t launch_publish_totals(const unsigned long long *totals, const int32_t *flags, int64_t *out, hipStream_t s)
{
    hipLaunchKernelGGL(k_publish_totals, dim3(1), dim3(WAVE), 0, s, totals, flags, out);
    return hipGetLastError();
}

// ------------------------------------------------------------- HLL sketch
// Registers of the rows in flight sit in LDS as 32-bit words (LDS has a
// 32-bit atomic max, Section 3.1 "parallel updates ... atomicMax"); they are
// packed to one byte per register (Section 4.3) when the sketch is stored.
// A row of SK_LONG or more entries is left to the whole workgroup, which takes the long rows of a turn one
// after the other once the lane groups are through with the short ones: on a power-law matrix the longest
// row, walked by one group of 16 lanes, was most of the kernel's time (R-MAT: 0.77 ms).  "Long" is relative: a row
// of long_from entries or more, which the launcher sets to 1024 or eight times the average row, whichever is more
// (where every row is long, sixteen groups side by side are 6 - 12 % faster than the workgroup on one row at a time).
constexpr int SK_LONG = 1024;
template <int M>
__global__ void __launch_bounds__(TPB)
k_hll_sketch(const int64_t *__restrict__ rp, const int32_t *__restrict__ col, int64_t rows, int g_log2,
             int64_t long_from, uint8_t *__restrict__ out)
{
    extern __shared__ uint32_t s_regs[];  // [TPB >> g_log2][M]
    __shared__ uint32_t s_big[M];
    __shared__ long long s_long[TPB / 8];   // (at most TPB / 8 rows per turn: groups have 8 lanes or more)
    __shared__ int s_nlong;
    constexpr int P = (M == 32) ? 5 : (M == 64) ? 6 : 7;
    const int G = 1 << g_log2;
    const int sub = threadIdx.x & (G - 1);
    const int rl = threadIdx.x >> g_log2;
    const int R = TPB >> g_log2;
    uint32_t *my = s_regs + rl * M;
    auto add = [&](uint32_t *regs, int32_t c) {
        const uint32_t h = hll_hash(c);
        const uint32_t w = h >> P;
        const uint32_t rank = w ? (uint32_t)(__clz((int)w) - P + 1) : (uint32_t)(32 - P + 1);
        atomicMax(&regs[h & (M - 1)], rank);
    };
    auto store = [&](const uint32_t *regs, int64_t row, int first, int step) {
        uint32_t *dst = reinterpret_cast<uint32_t *>(out + row * M);
        for (int j = first; j < M / 4; j += step)
            dst[j] = regs[4 * j] | (regs[4 * j + 1] << 8) | (regs[4 * j + 2] << 16) | (regs[4 * j + 3] << 24);
    };
    for (int64_t base = (int64_t)blockIdx.x * R; base < rows; base += (int64_t)gridDim.x * R) {   // uniform
        const int64_t row = base + rl;
        if (threadIdx.x == 0) s_nlong = 0;
        for (int j = sub; j < M; j += G) my[j] = 0;
        __syncthreads();
        bool mine = false;
        if (row < rows) {
            const int64_t p0 = rp[row], p1 = rp[row + 1];
            mine = p1 - p0 < long_from;
            if (!mine && sub == 0) s_long[atomicAdd(&s_nlong, 1)] = row;
            // four column ids per lane and turn (unconditional reads, index clamped): a long row is bound by
            // the latency of one load after the other otherwise
            for (int64_t p = p0 + sub; mine && p < p1; p += 4 * (int64_t)G) {
                int32_t c[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t q = p + (int64_t)i * G;
                    c[i] = col[q < p1 ? q : p1 - 1];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (p + (int64_t)i * G < p1) add(my, c[i]);
            }
        }
        wave_sync();
        if (mine) store(my, row, sub, G);
        __syncthreads();
        const int nlong = s_nlong;
        for (int i = 0; i < nlong; ++i) {   // uniform
            const int64_t lrow = s_long[i];
            for (int j = threadIdx.x; j < M; j += TPB) s_big[j] = 0;
            __syncthreads();
            const int64_t p1 = rp[lrow + 1];
            for (int64_t p = rp[lrow] + threadIdx.x; p < p1; p += 4 * (int64_t)TPB) {
                int32_t c[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int64_t q = p + (int64_t)k * TPB;
                    c[k] = col[q < p1 ? q : p1 - 1];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (p + (int64_t)k * TPB < p1) add(s_big, c[k]);
            }
            __syncthreads();
            store(s_big, lrow, (int)threadIdx.x, TPB);
            __syncthreads();
        }
        __syncthreads();   // (everyone has read s_nlong before the next turn clears it)
    }
}

// lanes_div: 1, or 4 when the rows are known to be of similar lengths - a lane keeps four entries in flight, so a
// quarter of the lanes per row puts four times the rows in flight (short rows are bound by the latency of their
// chain of loads); with skewed lengths the long rows then keep their few lanes busy long after the others.
hipError_t launch_hll_sketch(const Csr &B, int m, uint8_t *sketches, int lanes_div, hipStream_t s)
{
    if (B.rows == 0) return hipSuccess;
    const double avg = (double)B.nnz / (double)B.rows;
    const int g_log2 = ilog2_ceil(avg / (double)lanes_div, 3, 6);
    const int R = TPB >> g_log2;
    int64_t blocks = (B.rows + R - 1) / R;
    if (blocks > 256 * 64) blocks = 256 * 64;
    const size_t lds = (size_t)R * m * sizeof(uint32_t);
    const int64_t long_from = 8.0 * avg > (double)SK_LONG ? (int64_t)(8.0 * avg) : (int64_t)SK_LONG;
    switch (m) {
    case 32: hipLaunchKernelGGL(k_hll_sketch<32>, dim3((unsigned)blocks), dim3(TPB), lds, s, B.rp, B.col, B.rows, g_log2, long_from, sketches); break;
    case 64: hipLaunchKernelGGL(k_hll_sketch<64>, dim3((unsigned)blocks), dim3(TPB), lds, s, B.rp, B.col, B.rows, g_log2, long_from, sketches); break;
    case 128: hipLaunchKernelGGL(k_hll_sketch<128>, dim3((unsigned)blocks), dim3(TPB), lds, s, B.rp, B.col, B.rows, g_log2, long_from, sketches); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// -------------------------------------------------------------- HLL merge
// Registers are below 128, so a byte-wise maximum of eight registers is a few
// 64-bit integer operations: (a|0x80)-b keeps bit 7 of a byte set exactly
// when a >= b, and no borrow crosses a byte.
__device__ __forceinline__ uint64_t bytemax8(uint64_t a, uint64_t b)
{
    const uint64_t H = 0x8080808080808080ull;
    const uint64_t ge = (((a | H) - b) & H) >> 7;
    const uint64_t mask = ge * 0xFFull;
    return (a & mask) | (b & ~mask);
}

__device__ __forceinline__ double hll_alpha(int m)
{
    return m == 32 ? 0.697 : m == 64 ? 0.709 : 0.7213 / (1.0 + 1.079 / (double)m);
}

// One group of G lanes per selected row of A; L = M/8 lanes cover one sketch
// (8 registers per lane in a 64-bit word) so G/L entries of the row are
// merged at once.  Each 64-byte sketch of B is read as one coalesced line.
// A row of MG_LONG or more entries is left to the whole workgroup (TPB / L entries at once), which takes the
// long rows of its groups one after the other: on a power-law matrix a sampled row of tens of thousands of
// entries, merged by one group, was most of the sampled merge's time.  "Long" is long_from entries or more: 2048
// or eight times the average row of A, whichever is more (see k_hll_sketch).
constexpr int MG_LONG = 2048;
template <int M>
__global__ void __launch_bounds__(TPB)
k_hll_merge(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
            const uint64_t *__restrict__ sk, const int64_t *__restrict__ rows, int64_t n_rows, int g_log2,
            int64_t long_from, const int64_t *__restrict__ prod, const int32_t *__restrict__ maxb, const int64_t *__restrict__ b_rp,
            int64_t b_cols, double *__restrict__ est, uint64_t *__restrict__ merged)
{
    constexpr int L = M / 8;
    __shared__ long long s_long[TPB / L];   // (slot of the row, i.e. its position among the selected rows)
    __shared__ int s_nlong;
    __shared__ uint64_t s_acc[TPB];
    __shared__ long long s_blen[TPB / L];
    const int G = 1 << g_log2;  // >= L
    const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t t = gt >> g_log2;
    const int sub = (int)(gt & (G - 1));
    if (threadIdx.x == 0) s_nlong = 0;
    __syncthreads();
    // entries first, first + step, ... of a row, for this lane's slice of the sketch: four per lane and turn
    // (unconditional reads, index clamped; merging a sketch twice is harmless), so that the dependent loads
    // entry -> sketch of four entries overlap
    auto walk = [&](int64_t row, int slice, int first, int step, uint64_t &acc, long long &blen_max) {
        const int64_t e1 = a_rp[row + 1];
        for (int64_t e = a_rp[row] + first; e < e1; e += 4 * (int64_t)step) {
            int64_t k[4];
            uint64_t word[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t q = e + (int64_t)i * step;
                k[i] = a_col[q < e1 ? q : e1 - 1];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) word[i] = sk[k[i] * L + slice];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc = bytemax8(acc, word[i]);
            if (b_rp != nullptr && slice == 0) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const long long len = b_rp[k[i] + 1] - b_rp[k[i]];
                    blen_max = len > blen_max ? len : blen_max;
                }
            }
        }
    };
    // L consecutive lanes hold the merged sketch of slot t2 (row row2), 8 registers each: estimate and store
    auto finish = [&](uint64_t acc, long long blen_max, int64_t t2, int64_t row2, int slice, bool first_part) {
        double ssum = 0.0;
        int zeros = 0;
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const unsigned r = (unsigned)(acc >> (8 * b)) & 0xFFu;
            ssum += __longlong_as_double((long long)(1023 - (int)r) << 52);  // 2^-r, exact
            zeros += (r == 0);
        }
        for (int off = L >> 1; off > 0; off >>= 1) {
            ssum += __shfl_xor(ssum, off, WAVE);
            zeros += __shfl_xor(zeros, off, WAVE);
        }
        if (t2 < n_rows && first_part) {
            if (merged != nullptr) merged[t2 * L + slice] = acc;
            if (slice == 0) {
                const double dm = (double)M;
                double e = hll_alpha(M) * dm * dm / ssum;
                if (e <= 2.5 * dm && zeros > 0) e = dm * log(dm / (double)zeros);
                if (prod != nullptr) {
                    const long long pr = prod[row2];
                    const double hi = (double)(pr < b_cols ? pr : b_cols);
                    const double lo = (double)(maxb != nullptr ? (long long)maxb[row2] : blen_max);
                    e = e < lo ? lo : e;
                    e = e > hi ? hi : e;
                }
                est[t2] = e;
            }
        }
    };
    const int slice = sub & (L - 1);
    const int part = sub / L;
    const int parts = G / L;
    uint64_t acc = 0;
    long long blen_max = 0;
    int64_t row = -1;
    bool mine = false;
    if (t < n_rows) {
        row = rows ? rows[t] : t;
        mine = a_rp[row + 1] - a_rp[row] < long_from;
        if (mine) walk(row, slice, part, parts, acc, blen_max);
        else if (sub == 0) s_long[atomicAdd(&s_nlong, 1)] = t;
    }
    for (int off = L; off < G; off <<= 1) acc = bytemax8(acc, __shfl_xor((unsigned long long)acc, off, WAVE));
    if (b_rp != nullptr) blen_max = group_reduce_max(blen_max, G);
    finish(acc, blen_max, mine ? t : n_rows, row, slice, part == 0);
    __syncthreads();
    const int nlong = s_nlong;
    for (int i = 0; i < nlong; ++i) {   // uniform
        const int64_t t2 = s_long[i];
        const int64_t row2 = rows ? rows[t2] : t2;
        const int wslice = (int)threadIdx.x & (L - 1), wpart = (int)threadIdx.x / L;
        uint64_t a2 = 0;
        long long b2 = 0;
        walk(row2, wslice, wpart, TPB / L, a2, b2);
        s_acc[threadIdx.x] = a2;
        if (wslice == 0) s_blen[wpart] = b2;
        __syncthreads();
        // the first L lanes fold the partial sketches of the TPB / L parts
        uint64_t f = 0;
        long long fb = 0;
        if (threadIdx.x < L) {
            for (int p = 0; p < TPB / L; ++p) {
                f = bytemax8(f, s_acc[p * L + threadIdx.x]);
                fb = s_blen[p] > fb ? s_blen[p] : fb;
            }
        }
        if (threadIdx.x < WAVE) finish(f, fb, threadIdx.x < L ? t2 : n_rows, row2, (int)threadIdx.x & (L - 1), true);   // (whole first wave: lane swaps)
        __syncthreads();
    }
}

hipError_t launch_hll_merge(const Csr &A, const uint8_t *sketches, int m, const int64_t *rows, int64_t n_rows,
                            const int64_t *prod, const int32_t *maxb, const int64_t *b_rp, int64_t b_cols,
                            double *est, uint8_t *merged, int lanes_div, hipStream_t s)
{
    if (n_rows == 0) return hipSuccess;
    const int L = m / 8;
    const double avg = A.rows ? (double)A.nnz / (double)A.rows : 1.0;
    int g_log2 = ilog2_ceil(avg * L / (double)lanes_div, 0, 6);   // (lanes_div: see launch_hll_sketch)
    while ((1 << g_log2) < L) ++g_log2;
    const int64_t threads = n_rows << g_log2;
    const int64_t blocks = (threads + TPB - 1) / TPB;
    const uint64_t *sk = reinterpret_cast<const uint64_t *>(sketches);
    uint64_t *mg = reinterpret_cast<uint64_t *>(merged);
    const int64_t long_from = 8.0 * avg > (double)MG_LONG ? (int64_t)(8.0 * avg) : (int64_t)MG_LONG;
    switch (m) {
    case 32: hipLaunchKernelGGL(k_hll_merge<32>, dim3((unsigned)blocks), dim3(TPB), 0, s, A.rp, A.col, sk, rows, n_rows, g_log2, long_from, prod, maxb, b_rp, b_cols, est, mg); break;
    case 64: hipLaunchKernelGGL(k_hll_merge<64>, dim3((unsigned)blocks), dim3(TPB), 0, s, A.rp, A.col, sk, rows, n_rows, g_log2, long_from, prod, maxb, b_rp, b_cols, est, mg); break;
    case 128: hipLaunchKernelGGL(k_hll_merge<128>, dim3((unsigned)blocks), dim3(TPB), 0, s, A.rp, A.col, sk, rows, n_rows, g_log2, long_from, prod, maxb, b_rp, b_cols, est, mg); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------- row spans
// Column range that a row of C can reach: from the first entry of the rows of B it references to their last
// entry (B's rows in column order; where they are not, the range is only a guess, and the kernel that relies
// on it checks every product against it).  Used to choose the dense accumulator for rows whose range fits it
// (Section 3.3, accumulator selection).  One lane group per row as in k_row_products; rows of A with more than
// 64 entries per lane of the group are left with the full range (they are heavy rows, which have a dense
// accumulator of their own).  rows: list of row ids, or null for all rows 0 .. n-1; outputs indexed like rows.
__global__ void __launch_bounds__(TPB)
k_row_spans(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const int64_t *__restrict__ b_rp,
            const int32_t *__restrict__ b_col, const int64_t *__restrict__ rows, int64_t n, int g_log2,
            int32_t *__restrict__ cmin, int32_t *__restrict__ cmax)
{
    const int G = 1 << g_log2;
    const int R = TPB >> g_log2;
    const int rl = threadIdx.x >> g_log2;
    const int sub = threadIdx.x & (G - 1);
    for (int64_t base = (int64_t)blockIdx.x * R; base < n; base += (int64_t)gridDim.x * R) {
        const int64_t t = base + rl;
        int lo = 0x7fffffff, hi = -1;
        bool whole = false;
        if (t < n) {
            const int64_t row = rows ? rows[t] : t;
            const int64_t e0 = a_rp[row], e1 = a_rp[row + 1];
            whole = e1 - e0 > (int64_t)G * 64;
            if (!whole) {
                for (int64_t e = e0 + sub; e < e1; e += 4 * G) {
                    int64_t p0[4], p1[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int64_t idx = e + (int64_t)i * G;
                        const int32_t k = a_col[idx < e1 ? idx : e];
                        p0[i] = b_rp[k];
                        p1[i] = b_rp[k + 1];
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (e + (int64_t)i * G < e1 && p1[i] > p0[i]) {
                            const int32_t first = b_col[p0[i]], last = b_col[p1[i] - 1];
                            lo = first < lo ? first : lo;
                            hi = last > hi ? last : hi;
                        }
                    }
                }
            }
        }
        lo = -group_reduce_max(-lo, G);
        hi = group_reduce_max(hi, G);
        if (t < n && sub == 0) {
            cmin[t] = whole ? 0 : lo;
            cmax[t] = whole ? 0x7fffffff : hi;   // (hi < lo: a row without products)
        }
    }
}

hipError_t launch_row_spans(const Csr &A, const Csr &B, const int64_t *rows, int64_t n, int32_t *cmin, int32_t *cmax,
                            hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const double avg = A.rows ? (double)A.nnz / (double)A.rows : 0.0;
    const int g_log2 = ilog2_ceil(avg / 4.0, 1, 6);
    const int R = TPB >> g_log2;
    int64_t blocks = (n + R - 1) / R;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_row_spans, dim3((unsigned)blocks), dim3(TPB), 0, s, A.rp, A.col, B.rp, B.col, rows, n, g_log2,
                       cmin, cmax);
    return hipGetLastError();
}

// ----------------------------------------------------------- sample rows
// The stratified sample of Section 3.2 (one row out of each of ns equal strata, chosen by a hash of the
// stratum's number and the seed), written on the device: the same rows as the host helper behind
// ocean_sample_rows gives.
__global__ void __launch_bounds__(TPB)
k_sample_rows(int64_t rows, int64_t ns, uint32_t seed, int64_t *__restrict__ out)
{
    const int64_t t = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (t >= ns) return;
    const int64_t lo = (int64_t)((unsigned __int128)t * (unsigned __int128)rows / (unsigned __int128)ns);
    const int64_t hi = (int64_t)((unsigned __int128)(t + 1) * (unsigned __int128)rows / (unsigned __int128)ns);
    const uint32_t h = fmix32(seed + 0x9E3779B9u * (uint32_t)(t + 1));
    out[t] = lo + (int64_t)(h % (uint64_t)(hi - lo));
}

hipError_t launch_sample_rows(int64_t rows, int64_t ns, uint32_t seed, int64_t *out, hipStream_t s)
{
    if (ns <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_sample_rows, dim3((unsigned)((ns + TPB - 1) / TPB)), dim3(TPB), 0, s, rows, ns, seed, out);
    return hipGetLastError();
}

// --------------------------------------------------------- sample reduce
// Sums over the sampled rows in a fixed order (one workgroup, strided partial
// sums, tree reduction), so the sampled CR is the same on every run.
// out[0] = sum of products, out[1] = sum of estimates (their ratio is the sampled CR, Section 3.2);
// out[2], out[3] = sum and sum of squares of the per-row ratios products / estimate, out[4] = rows counted
// (mean and standard deviation of the compression ratio over the sample, Section 4.1); out[5] = sampled rows
// whose column range is narrow enough for the dense accumulator to pay (cmin / cmax of the sampled rows given).
constexpr int SR_THREADS = 1024;
__global__ void __launch_bounds__(SR_THREADS)
k_sample_reduce(const int64_t *__restrict__ rows, int64_t n_rows, const int64_t *__restrict__ prod,
                const double *__restrict__ est, const int32_t *__restrict__ cmin, const int32_t *__restrict__ cmax,
                int64_t n_cols, int vbytes, double bound_coef, double *out)
{
    constexpr int NS = 6;
    __shared__ double s_acc[NS][SR_THREADS];
    double acc[NS] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    // four sampled rows per thread and turn, their dependent loads (row id -> products) issued together
    for (int64_t t0 = threadIdx.x; t0 < n_rows; t0 += 4 * SR_THREADS) {
        double e[4];
        int64_t r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t t = t0 + (int64_t)i * SR_THREADS;
            e[i] = t < n_rows ? est[t] : 0.0;
            r[i] = rows[t < n_rows ? t : t0];
        }
        double p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = (double)prod[r[i]];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (e[i] > 0.0) {
                const double q = p[i] / e[i];
                acc[0] += p[i]; acc[1] += e[i]; acc[2] += q; acc[3] += q * q; acc[4] += 1.0;
                if (cmin != nullptr) {
                    const int64_t t = t0 + (int64_t)i * SR_THREADS;
                    const long long span = (long long)cmax[t] - (long long)cmin[t] + 1;
                    const double ub = p[i] < (double)n_cols ? p[i] : (double)n_cols;
                    long long slots = 16;
                    while ((double)slots < bound_coef * ub && slots < (1ll << 40)) slots <<= 1;   // table from the bound
                    if (dense_span_pays(span, slots, vbytes)) acc[5] += 1.0;
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < NS; ++k) s_acc[k][threadIdx.x] = acc[k];
    __syncthreads();
    for (int off = SR_THREADS / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) {
#pragma unroll
            for (int k = 0; k < NS; ++k) s_acc[k][threadIdx.x] += s_acc[k][threadIdx.x + off];
        }
        __syncthreads();
    }
    if (threadIdx.x < NS) out[threadIdx.x] = s_acc[threadIdx.x][0];
}

hipError_t launch_sample_reduce(const int64_t *rows, int64_t n_rows, const int64_t *prod, const double *est,
                                const int32_t *cmin, const int32_t *cmax, int64_t n_cols, int vbytes, double bound_coef,
                                double *out, hipStream_t s)
{
    hipLaunchKernelGGL(k_sample_reduce, dim3(1), dim3(SR_THREADS), 0, s, rows, n_rows, prod, est, cmin, cmax, n_cols,
                       vbytes, bound_coef, out);
    return hipGetLastError();
}

}  // namespace ocean
