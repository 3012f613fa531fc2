// Binning (paper Sections 2.3, 3.2, 5.3): turn a per-row size prediction into a
// hash-table size, a kernel configuration ("bin") and an output capacity,
// group row ids per bin, and the prefix sums that place rows in memory.
#include "ocean_internal.hpp"

namespace ocean {

constexpr int TPB = 256;

struct BinTable {
    int n;
    int32_t slots[OCEAN_MAX_BINS];
};

// need = table slots the row asks for, cap = output entries reserved for it.
//   mode 0  upper bound: cap = ub = min(prod, n), need = ceil(bound_coef * ub)   (Section 3.2, upper-bound workflow)
//   (in modes 1 and 2 the table is limited to ceil(bound_coef * ub) slots as well: more cannot be of use)
//   mode 1  estimate:    cap = ceil(coef * scale * est), need = ceil(table_coef * scale * est), both limited to ub
//                        (Section 5.3: estimate x coefficient; table_coef <= coef)
//   mode 2  exact:       cap = nnz, need = ceil(coef * nnz) limited to ub   (two-pass workflow)
//   mode 3  symbolic:    need = ceil(1.25 * e), no capacity; e = ub, or with assisted binning (coef > 1,
//                        Section 4.1) ceil(prod / coef) kept inside [longest referenced row of B, ub]
// max_cap receives the largest capacity among the rows of the last (global-memory) bin.
__global__ void __launch_bounds__(TPB)
k_classify(int64_t m, int mode, double coef, double table_coef, double bound_coef, double scale, BinTable bt, int64_t n_cols,
           const int64_t *__restrict__ prod, const double *__restrict__ est, const int32_t *__restrict__ nnz_exact,
           const int32_t *__restrict__ row_mask, const int32_t *__restrict__ lower_bound,
           const int32_t *__restrict__ cmin, const int32_t *__restrict__ cmax, int vbytes,
           uint8_t *__restrict__ bin_of_row, int32_t *__restrict__ cap,
           unsigned long long *bin_count, unsigned long long *bin_prod, unsigned long long *max_cap)
{
    __shared__ unsigned int s_cnt[OCEAN_MAX_BINS];
    __shared__ unsigned long long s_prod[OCEAN_MAX_BINS];
    __shared__ unsigned int s_maxcap;
    if (threadIdx.x < OCEAN_MAX_BINS) { s_cnt[threadIdx.x] = 0; s_prod[threadIdx.x] = 0ull; }
    if (threadIdx.x == 0) s_maxcap = 0;
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x; i < m; i += (int64_t)gridDim.x * TPB) {
        int bin = BIN_NONE;
        long long c = 0;
        const bool active = (row_mask == nullptr) || (row_mask[i] < 0);
        const long long pr = prod[i];
        const long long ub = pr < n_cols ? pr : n_cols;
        if (active && ub > 0) {
            long long need;
            // the most slots a row can make use of: its bound with the load factor of bound-sized tables
            const long long ub_slots = bound_coef > 1.0 ? (long long)ceil(bound_coef * (double)ub) : ub;
            if (mode == 0) {
                c = ub;
                need = ub_slots;
            } else if (mode == 1) {
                double want = ceil(coef * scale * est[i]);
                c = want >= (double)ub ? ub : (long long)want;
                if (c < 1) c = 1;
                double slots = ceil(table_coef * scale * est[i]);
                need = slots >= (double)ub_slots ? ub_slots : (long long)slots;
                if (need < 1) need = 1;
            } else if (mode == 2) {
                c = nnz_exact[i];
                double want = ceil(coef * (double)c);
                need = want >= (double)ub_slots ? ub_slots : (long long)want;
                if (need < c) need = c;
            } else {
                long long e = ub;
                if (coef > 1.0) {
                    const double q = ceil((double)pr / coef);
                    e = q >= (double)ub ? ub : (long long)q;
                    if (lower_bound != nullptr && e < (long long)lower_bound[i]) e = lower_bound[i];
                    if (e > ub) e = ub;
                    if (e < 1) e = 1;
                }
                need = e + (e + 3) / 4;
            }
            bin = bt.n - 1;
            for (int b = 0; b < bt.n; ++b)
                if ((long long)bt.slots[b] >= need) { bin = b; break; }
            if (cmin != nullptr) {
                // Section 3.3, accumulator selection: the dense accumulator over the row's own column range where
                // it needs no more memory than the hash table the row would get
                const long long span = (long long)cmax[i] - (long long)cmin[i] + 1;
                if (dense_span_pays(span, (long long)bt.slots[bin], vbytes)) {
                    bin = NB_DSPAN;
                    if (c > span) c = span;
                }
            }
            atomicAdd(&s_cnt[bin], 1u);
            if (bin_prod != nullptr) atomicAdd(&s_prod[bin], (unsigned long long)pr);
            if (bin == bt.n - 1 && c > 0) atomicMax(&s_maxcap, (unsigned int)c);
        }
        bin_of_row[i] = (uint8_t)bin;
        if (cap != nullptr) cap[i] = (int32_t)c;
    }
    __syncthreads();
    if (threadIdx.x < OCEAN_MAX_BINS && s_cnt[threadIdx.x]) atomicAdd(&bin_count[threadIdx.x], (unsigned long long)s_cnt[threadIdx.x]);
    if (bin_prod != nullptr && threadIdx.x < OCEAN_MAX_BINS && s_prod[threadIdx.x]) atomicAdd(&bin_prod[threadIdx.x], s_prod[threadIdx.x]);
    if (threadIdx.x == 0 && s_maxcap && max_cap != nullptr) atomicMax(max_cap, (unsigned long long)s_maxcap);
}

hipError_t launch_classify(int64_t m, const BinParams &p, double scale, const int64_t *prod, const double *est,
                           const int32_t *nnz_exact, const int32_t *row_mask, const int32_t *lower_bound,
                           uint8_t *bin_of_row, int32_t *cap, unsigned long long *bin_count,
                           unsigned long long *bin_prod, unsigned long long *max_cap, hipStream_t s)
{
    static_assert(NB_ALL <= OCEAN_MAX_BINS, "the dense-range bin has a place in the per-bin arrays");
    if (m == 0) return hipSuccess;
    BinTable bt;
    bt.n = p.n_bins;
    for (int b = 0; b < OCEAN_MAX_BINS; ++b) bt.slots[b] = b < p.n_bins ? p.slots[b] : 0;
    int64_t blocks = (m + TPB - 1) / TPB;
    if (blocks > 1024) blocks = 1024;   // one set of atomics per workgroup: keep the workgroups few
    hipLaunchKernelGGL(k_classify, dim3((unsigned)blocks), dim3(TPB), 0, s, m, p.mode, p.coef, (p.table_coef > 0.0 && p.table_coef < p.coef) ? p.table_coef : p.coef, p.bound_coef, scale, bt, p.n_cols,
                       prod, est, nnz_exact, row_mask, lower_bound, p.mode != 3 ? p.cmin : nullptr, p.cmax, p.vbytes, bin_of_row,
                       cap, bin_count, bin_prod, max_cap);
    return hipGetLastError();
}

// Row ids grouped by bin: bin b occupies bin_rows[prefix(b) .. prefix(b)+count(b)).  A workgroup
// counts its rows per bin in LDS, claims one contiguous range per bin, then fills it.
constexpr int SC_ITEMS = 8;
__global__ void __launch_bounds__(TPB)
k_scatter(int64_t m, int n_bins, const uint8_t *__restrict__ bin_of_row,
          const unsigned long long *__restrict__ bin_count, unsigned long long *bin_cursor,
          int32_t *__restrict__ bin_rows)
{
    __shared__ unsigned int s_cnt[OCEAN_MAX_BINS];
    __shared__ unsigned long long s_base[OCEAN_MAX_BINS];
    if (threadIdx.x < OCEAN_MAX_BINS) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    const int64_t tile = (int64_t)blockIdx.x * TPB * SC_ITEMS;
    int bin[SC_ITEMS];
    unsigned int rank[SC_ITEMS];
#pragma unroll
    for (int q = 0; q < SC_ITEMS; ++q) {
        const int64_t i = tile + (int64_t)q * TPB + threadIdx.x;
        bin[q] = BIN_NONE;
        rank[q] = 0;
        if (i < m) {
            bin[q] = bin_of_row[i];
            if (bin[q] != BIN_NONE) rank[q] = atomicAdd(&s_cnt[bin[q]], 1u);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < n_bins) {
        unsigned long long start = 0;
        for (int b = 0; b < (int)threadIdx.x; ++b) start += bin_count[b];
        unsigned long long off = s_cnt[threadIdx.x] ? atomicAdd(&bin_cursor[threadIdx.x], (unsigned long long)s_cnt[threadIdx.x]) : 0ull;
        s_base[threadIdx.x] = start + off;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < SC_ITEMS; ++q) {
        const int64_t i = tile + (int64_t)q * TPB + threadIdx.x;
        if (bin[q] != BIN_NONE) bin_rows[s_base[bin[q]] + rank[q]] = (int32_t)i;
    }
}

hipError_t launch_scatter(int64_t m, int n_bins, const uint8_t *bin_of_row, const unsigned long long *bin_count,
                          unsigned long long *bin_cursor, int32_t *bin_rows, hipStream_t s)
{
    if (m == 0) return hipSuccess;
    const int64_t blocks = (m + TPB * SC_ITEMS - 1) / (TPB * SC_ITEMS);
    hipLaunchKernelGGL(k_scatter, dim3((unsigned)blocks), dim3(TPB), 0, s, m, n_bins, bin_of_row, bin_count,
                       bin_cursor, bin_rows);
    return hipGetLastError();
}

// ------------------------------------------------------------------ scan
// Exclusive prefix sum int32 -> int64 with n+1 outputs (out[n] = total), in
// three launches: per-block sums, scan of the block sums, per-block scan.
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = TPB * SCAN_ITEMS;

int64_t scan_tmp_elems(int64_t n) { return (n + SCAN_TILE - 1) / SCAN_TILE + 1; }

__device__ __forceinline__ long long block_exclusive_scan(long long v, long long *s_wave, long long &total)
{
    // inclusive scan inside the wave
    long long inc = v;
    for (int off = 1; off < WAVE; off <<= 1) {
        long long o = __shfl_up(inc, off, WAVE);
        if (lane_id() >= off) inc += o;
    }
    const int w = threadIdx.x / WAVE;
    if (lane_id() == WAVE - 1) s_wave[w] = inc;
    __syncthreads();
    long long wave_off = 0, tot = 0;
    for (int i = 0; i < TPB / WAVE; ++i) {
        if (i < w) wave_off += s_wave[i];
        tot += s_wave[i];
    }
    __syncthreads();
    total = tot;
    return wave_off + inc - v;
}

__global__ void __launch_bounds__(TPB)
k_scan_block_sums(const int32_t *__restrict__ in, int64_t n, int64_t *__restrict__ block_sum)
{
    __shared__ long long s_wave[TPB / WAVE];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    long long v = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (base + k < n) v += in[base + k];
    long long total;
    block_exclusive_scan(v, s_wave, total);
    if (threadIdx.x == 0) block_sum[blockIdx.x] = total;
}

__global__ void __launch_bounds__(TPB)
k_scan_of_sums(int64_t *block_sum, int64_t n_blocks, unsigned long long *total_out)
{
    __shared__ long long s_wave[TPB / WAVE];
    long long carry = 0;
    for (int64_t base = 0; base < n_blocks; base += TPB) {
        const int64_t i = base + threadIdx.x;
        long long v = i < n_blocks ? block_sum[i] : 0;
        long long total;
        long long ex = block_exclusive_scan(v, s_wave, total);
        if (i < n_blocks) block_sum[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) {
        block_sum[n_blocks] = carry;
        if (total_out != nullptr) *total_out = (unsigned long long)carry;
    }
}

// The whole scan by one workgroup, tile after tile with a running carry: for inputs so short that three
// launches would cost more than the work (up to SCAN_SMALL_MAX elements).
constexpr int64_t SCAN_SMALL_MAX = 65536;
__global__ void __launch_bounds__(TPB)
k_scan_small(const int32_t *__restrict__ in, int64_t n, int64_t *__restrict__ out, unsigned long long *total_out)
{
    __shared__ long long s_wave[TPB / WAVE];
    long long carry = 0;
    for (int64_t tile = 0; tile < n; tile += SCAN_TILE) {
        const int64_t base = tile + (int64_t)threadIdx.x * SCAN_ITEMS;
        long long item[SCAN_ITEMS];
        long long v = 0;
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            item[k] = (base + k < n) ? in[base + k] : 0;
            v += item[k];
        }
        long long total;
        long long run = carry + block_exclusive_scan(v, s_wave, total);
#pragma unroll
        for (int k = 0; k < SCAN_ITEMS; ++k) {
            if (base + k < n) out[base + k] = run;
            run += item[k];
        }
        carry += total;
    }
    if (threadIdx.x == 0) {
        out[n] = carry;
        if (total_out != nullptr) *total_out = (unsigned long long)carry;
    }
}

__global__ void __launch_bounds__(TPB)
k_scan_apply(const int32_t *__restrict__ in, int64_t n, const int64_t *__restrict__ block_sum, int64_t n_blocks,
             int64_t *__restrict__ out)
{
    __shared__ long long s_wave[TPB / WAVE];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    long long item[SCAN_ITEMS];
    long long v = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        item[k] = (base + k < n) ? in[base + k] : 0;
        v += item[k];
    }
    long long total;
    long long run = block_sum[blockIdx.x] + block_exclusive_scan(v, s_wave, total);
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (base + k < n) out[base + k] = run;
        run += item[k];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out[n] = block_sum[n_blocks];
}

// total_out (may be null): a device word that receives the sum of all elements as well.
hipError_t launch_scan_i32_to_i64(const int32_t *in, int64_t n, int64_t *out, int64_t *block_tmp,
                                  unsigned long long *total_out, hipStream_t s)
{
    const int64_t n_blocks = (n + SCAN_TILE - 1) / SCAN_TILE;
    if (n <= SCAN_SMALL_MAX) {   // (also n == 0: out[0] = 0)
        hipLaunchKernelGGL(k_scan_small, dim3(1), dim3(TPB), 0, s, in, n, out, total_out);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_scan_block_sums, dim3((unsigned)n_blocks), dim3(TPB), 0, s, in, n, block_tmp);
    hipLaunchKernelGGL(k_scan_of_sums, dim3(1), dim3(TPB), 0, s, block_tmp, n_blocks, total_out);
    hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)n_blocks), dim3(TPB), 0, s, in, n, block_tmp, n_blocks, out);
    return hipGetLastError();
}

// ------------------------------------------------------------ small fills
template <typename T>
__global__ void k_fill(T *p, int64_t n, T v)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

template <typename T>
static hipError_t fill(T *p, int64_t n, T v, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    int64_t blocks = (n + TPB * 4 - 1) / (TPB * 4);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_fill<T>, dim3((unsigned)blocks), dim3(TPB), 0, s, p, n, v);
    return hipGetLastError();
}
hipError_t launch_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t s) { return fill<int32_t>(p, n, v, s); }
hipError_t launch_fill_u64(unsigned long long *p, int64_t n, unsigned long long v, hipStream_t s) { return fill<unsigned long long>(p, n, v, s); }

// -------------------------------------------------- overflow bookkeeping
__global__ void __launch_bounds__(TPB)
k_count_overflow(int64_t m, const int32_t *__restrict__ row_nnz, unsigned long long *count)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    const bool ovf = i < m && row_nnz[i] < 0;
    const unsigned long long b = __ballot(ovf);
    if (b != 0 && lane_id() == 0) atomicAdd(count, (unsigned long long)__popcll(b));
}

hipError_t launch_count_overflow(int64_t m, const int32_t *row_nnz, unsigned long long *count, hipStream_t s)
{
    if (m == 0) return hipSuccess;
    hipLaunchKernelGGL(k_count_overflow, dim3((unsigned)((m + TPB - 1) / TPB)), dim3(TPB), 0, s, m, row_nnz, count);
    return hipGetLastError();
}

// final size of each row: first attempt unless it overflowed, then the retry's
__global__ void __launch_bounds__(TPB)
k_final_nnz(int64_t m, const int32_t *__restrict__ nnz1, const int32_t *__restrict__ nnz2, int32_t *__restrict__ out)
{
    const int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (i < m) out[i] = nnz1[i] >= 0 ? nnz1[i] : nnz2[i];
}

hipError_t launch_final_nnz(int64_t m, const int32_t *nnz1, const int32_t *nnz2, int32_t *out, hipStream_t s)
{
    if (m == 0) return hipSuccess;
    hipLaunchKernelGGL(k_final_nnz, dim3((unsigned)((m + TPB - 1) / TPB)), dim3(TPB), 0, s, m, nnz1, nnz2, out);
    return hipGetLastError();
}

// ------------------------------------------------------ per-bin work sums
// For reporting only: intermediate products, entries of A and entries of C
// handled by each numeric bin.  sums[3 * OCEAN_MAX_BINS], zero on entry.
__global__ void __launch_bounds__(TPB)
k_bin_work(int64_t m, const uint8_t *__restrict__ bin_of_row, const int64_t *__restrict__ prod,
           const int64_t *__restrict__ a_rp, const int32_t *__restrict__ row_nnz, unsigned long long *sums)
{
    __shared__ unsigned long long s_sum[3 * OCEAN_MAX_BINS];
    if (threadIdx.x < 3 * OCEAN_MAX_BINS) s_sum[threadIdx.x] = 0;
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * TPB + threadIdx.x; i < m; i += (int64_t)gridDim.x * TPB) {
        const int b = bin_of_row[i];
        if (b != BIN_NONE) {
            atomicAdd(&s_sum[b], (unsigned long long)prod[i]);
            atomicAdd(&s_sum[OCEAN_MAX_BINS + b], (unsigned long long)(a_rp[i + 1] - a_rp[i]));
            const int32_t c = row_nnz[i];
            if (c > 0) atomicAdd(&s_sum[2 * OCEAN_MAX_BINS + b], (unsigned long long)c);
        }
    }
    __syncthreads();
    if (threadIdx.x < 3 * OCEAN_MAX_BINS && s_sum[threadIdx.x]) atomicAdd(&sums[threadIdx.x], s_sum[threadIdx.x]);
}

hipError_t launch_bin_work(int64_t m, const uint8_t *bin_of_row, const int64_t *prod, const int64_t *a_rp,
                           const int32_t *row_nnz, unsigned long long *sums, hipStream_t s)
{
    if (m == 0) return hipSuccess;
    int64_t blocks = (m + TPB - 1) / TPB;
    if (blocks > 512) blocks = 512;
    hipLaunchKernelGGL(k_bin_work, dim3((unsigned)blocks), dim3(TPB), 0, s, m, bin_of_row, prod, a_rp,
                       row_nnz, sums);
    return hipGetLastError();
}

}  // namespace ocean
