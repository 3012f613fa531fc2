// Internal declarations shared by the HIP translation units of the library.
// gfx950 only: wave64, 160 KB LDS per workgroup, native LDS/global fp64 atomic add.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ocean_spgemm.h"

namespace ocean {

constexpr int WAVE = 64;
constexpr int32_t EMPTY_KEY = -1;          // column ids are >= 0
constexpr int32_t SORT_PAD = 0x7fffffff;   // sorts after every valid column id

// ---------------------------------------------------------------- bins ----
// Numeric bins (Section 4.3 uses five halving configurations plus a
// multi-short-row and a long-row one; the sizes here are re-derived for 160 KB
// of LDS and 64-wide waves).  slots = hash-table entries of the bin.
enum NumericBin {
    NB_E16 = 0,   // 16 slots: with sizes from the product bound, expand-sort-compress, 16 lanes per row (else as NB_G8)
    NB_G8,        // 8 lanes per row, 8 rows per wave, 32 slots (product bound: expand-sort-compress, 32 lanes per row)
    NB_G16,       // 16 lanes per row, 4 rows per wave, 64 slots
    NB_W64,       // one wave per row, 256 slots
    NB_S512,      // one workgroup per row from here on
    NB_S1K,
    NB_S2K,
    NB_S4K,
    NB_S8K,       // largest table with keys and values both in LDS
    NB_HYBRID,    // 32768 keys in LDS, values in a global slab (Section 3.3, enhanced hash accumulator)
    NB_GLOBAL,    // whole table in global memory
    NB_COUNT
};
constexpr int32_t kNumericSlots[NB_COUNT] = {16, 32, 64, 256, 512, 1024, 2048, 4096, 8192, 32768, 0x7fffffff};

enum SymbolicBin {
    SB_G16 = 0,   // 64 keys
    SB_W64,       // 256 keys
    SB_S1K,
    SB_S4K,
    SB_S16K,
    SB_S32K,      // 128 KB of keys
    SB_BITMAP,    // LDS bitmap over column windows
    SB_COUNT
};
constexpr int32_t kSymbolicSlots[SB_COUNT] = {64, 256, 1024, 4096, 16384, 32768, 0x7fffffff};

constexpr int32_t BIN_NONE = 255;          // row takes no part in this launch set

// Dense accumulator over a row's own column range (Section 3.3, accumulator selection: the kind that needs fewer
// resources, dense when both need the same): values and one presence bit per column of the range against keys
// and values of a hash table.  Rows of the 512-slot bin and beyond are candidates; the range must fit the
// kernel's LDS window.
constexpr int NB_DSPAN = NB_COUNT;          // index of that bin in the per-bin arrays (after the hash bins)
constexpr int NB_ALL = NB_COUNT + 1;
constexpr int64_t DS_MAX_COLS = 4096;
__host__ __device__ inline bool dense_span_pays(long long span, long long slots, int vbytes)
{
    return span > 0 && span <= DS_MAX_COLS && slots >= 512 && span * (8 * vbytes + 1) <= slots * 8 * (4 + vbytes);
}

// ------------------------------------------------------------- CSR view ----
struct Csr {
    const int64_t *rp;
    const int32_t *col;
    const void *val;
    int64_t rows, cols, nnz;
};

// ------------------------------------------------------ device helpers ----
#if defined(__HIPCC__)
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (WAVE - 1)); }

// Orders this wave's LDS/global accesses for the compiler; the hardware runs a
// wave's LDS instructions in issue order, so lanes of one wave see each
// other's earlier writes after this point.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ uint32_t fmix32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

// Hash used by the HLL sketches (the same function must build every sketch
// that is merged, Section 3.1).
__device__ __forceinline__ uint32_t hll_hash(int32_t col) { return fmix32((uint32_t)col + 0x9E3779B9u); }

// Fibonacci hashing for the accumulator tables: top `bits` bits of key * golden ratio.
__device__ __forceinline__ uint32_t table_hash(int32_t key, int bits)
{
    return ((uint32_t)key * 0x9E3779B1u) >> (32 - bits);
}

// Probe stride of a key (double hashing): odd, so it visits every slot of a
// power-of-two table.  A wave waits for its slowest lane, so what matters is
// the longest probe sequence among 64 concurrent insertions; linear probing's
// clustering makes that several times longer than with independent strides,
// and LDS has no locality that would reward neighbouring slots.
__device__ __forceinline__ uint32_t table_step(int32_t key, int bits)
{
    return ((((uint32_t)key * 0x85EBCA6Bu) >> (32 - bits)) << 1) | 1u;
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves, which
// cost a vector instruction each and no trip to LDS: shifts by 1, 2, 4 and 8 lanes inside the
// rows of 16 lanes, then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into the upper
// half.  A lane without a source adds 0.  Every lane of the wave must be active.
__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);   // row_bcast:15, rows 1 and 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);   // row_bcast:31, rows 2 and 3
    return v;
}
// The same inside every group of G = 8 or 16 consecutive lanes (sub = lane inside the group).
template <int G>
__device__ __forceinline__ uint32_t group_inclusive_scan_u32(uint32_t v, int sub)
{
    static_assert(G == 8 || G == 16, "groups inside one row of 16 lanes");
    uint32_t o;
    o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false); v += sub >= 1 ? o : 0u;
    o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false); v += sub >= 2 ? o : 0u;
    o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false); v += sub >= 4 ? o : 0u;
    if (G == 16) { o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false); v += sub >= 8 ? o : 0u; }
    return v;
}
// Sum over every group of G = 8 or 16 consecutive lanes, in each of its lanes (butterfly of
// lane swaps: neighbours, pairs, mirrored halves of 8, mirrored rows of 16).
template <int G>
__device__ __forceinline__ uint32_t group_sum_u32(uint32_t v)
{
    static_assert(G == 8 || G == 16, "groups inside one row of 16 lanes");
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);    // quad_perm [1,0,3,2]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false);    // quad_perm [2,3,0,1]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, false);   // row_half_mirror
    if (G == 16) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, false);   // row_mirror
    return v;
}
// Value of lane `l` (the same number in every lane) of v.
__device__ __forceinline__ uint32_t wave_read_lane_u32(uint32_t v, int l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, __builtin_amdgcn_readfirstlane(l));
}
// Sum over the wave, in every lane.
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v)
{
    return wave_read_lane_u32(wave_inclusive_scan_u32(v), WAVE - 1);
}
// Largest value over the wave, as a wave-uniform number: the moves of the prefix sum with max in place of
// add (a lane without a source keeps its own value), read from the last lane.  Every lane must be active.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    auto larger = [](uint32_t a, uint32_t b) { return a > b ? a : b; };
    v = larger(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false));   // row_shr:1
    v = larger(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false));   // row_shr:2
    v = larger(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false));   // row_shr:4
    v = larger(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false));   // row_shr:8
    v = larger(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false));   // row_bcast:15, rows 1 and 3
    v = larger(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false));   // row_bcast:31, rows 2 and 3
    return wave_read_lane_u32(v, WAVE - 1);
}
// Workgroup level of a two-level prefix sum: part[w] holds the sum of wave w (NW <= 64 waves).
// Returns the sum of the waves before `wave`; total = sum of all.  Every lane must be active.
template <int NW>
__device__ __forceinline__ uint32_t waves_before_u32(const uint32_t *part, int wave, uint32_t &total)
{
    static_assert(NW <= WAVE, "one lane per wave");
    const int lane = (int)(threadIdx.x & (WAVE - 1));
    const uint32_t inc = wave_inclusive_scan_u32(lane < NW ? part[lane] : 0u);
    total = wave_read_lane_u32(inc, NW - 1);
    const uint32_t upto = wave_read_lane_u32(inc, wave > 0 ? wave - 1 : 0);
    return wave > 0 ? upto : 0u;
}

template <typename T>
__device__ __forceinline__ T group_reduce_sum(T v, int width)
{
    for (int off = width >> 1; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}
template <typename T>
__device__ __forceinline__ T group_reduce_max(T v, int width)
{
    for (int off = width >> 1; off > 0; off >>= 1) {
        T o = __shfl_xor(v, off, WAVE);
        v = o > v ? o : v;
    }
    return v;
}
#endif

// Totals of the row-products pass are kept in ROW_TOTAL_SLOTS slots of ROW_TOTAL_STRIDE 64-bit words each (128
// bytes apart): [0] sum of products, [1] largest row, [2] products of the heavy rows; see analysis.hip.
constexpr int ROW_TOTAL_SLOTS = 32;
constexpr int ROW_TOTAL_STRIDE = 16;

// --------------------------------------------------- launcher prototypes ----
// analysis.hip
hipError_t launch_validate(const Csr &A, const Csr &B, int32_t *flags, unsigned long long *b_near_pairs, hipStream_t s);
hipError_t launch_row_products(const Csr &A, const int64_t *b_rp, int64_t b_rows, int64_t *prod, int32_t *maxb,
                               unsigned long long *totals, int32_t *flags, int32_t *long_rows,
                               unsigned long long *long_count, hipStream_t s);
hipError_t launch_publish_totals(const unsigned long long *totals, const int32_t *flags, int64_t *out, hipStream_t s);
hipError_t launch_hll_sketch(const Csr &B, int m, uint8_t *sketches, int lanes_div, hipStream_t s);
hipError_t launch_hll_merge(const Csr &A, const uint8_t *sketches, int m, const int64_t *rows, int64_t n_rows,
                            const int64_t *prod, const int32_t *maxb, const int64_t *b_rp, int64_t b_cols,
                            double *est, uint8_t *merged, int lanes_div, hipStream_t s);
hipError_t launch_sample_rows(int64_t rows, int64_t ns, uint32_t seed, int64_t *out, hipStream_t s);
hipError_t launch_row_spans(const Csr &A, const Csr &B, const int64_t *rows, int64_t n, int32_t *cmin, int32_t *cmax,
                            hipStream_t s);
hipError_t launch_sample_reduce(const int64_t *rows, int64_t n_rows, const int64_t *prod, const double *est,
                                const int32_t *cmin, const int32_t *cmax /*of the sampled rows, may be null*/,
                                int64_t n_cols, int vbytes, double bound_coef,
                                double *out /*[6]: sum prod, sum est, sum cr, sum cr^2, rows, rows a dense range pays for*/,
                                hipStream_t s);

// binning.hip
struct BinParams {
    int mode;            // 0 upper bound, 1 estimate, 2 exact nnz, 3 symbolic pass (see k_classify)
    double coef;         // table slots per predicted entry; mode 3: the compression ratio the product counts
                         // are divided by (assisted symbolic binning, Section 4.1), 1.0 = plain product counts
    double table_coef;   // mode 1: table slots per estimated entry when smaller than coef (0: coef itself); the
                         // reserved output stays coef x estimate
    double bound_coef;   // table slots per intermediate product beyond which a table is of no use (modes 0, 1, 2;
                         // at most 1.0 = the product bound itself)
    const int32_t *cmin; // per row: first and last column the row can reach (k_row_spans), or null: rows whose range
    const int32_t *cmax; // pays for it go to the dense-range bin NB_DSPAN (modes 0, 1, 2)
    int vbytes;          // bytes of a value (with cmin)
    int n_bins;
    int32_t slots[OCEAN_MAX_BINS];
    int64_t n_cols;
};
hipError_t launch_classify(int64_t m, const BinParams &p, double scale, const int64_t *prod, const double *est,
                           const int32_t *nnz_exact, const int32_t *row_mask, const int32_t *lower_bound,
                           uint8_t *bin_of_row, int32_t *cap, unsigned long long *bin_count,
                           unsigned long long *bin_prod /*products per bin, may be null*/, unsigned long long *max_cap,
                           hipStream_t s);
hipError_t launch_scatter(int64_t m, int n_bins, const uint8_t *bin_of_row, const unsigned long long *bin_count,
                          unsigned long long *bin_cursor, int32_t *bin_rows, hipStream_t s);
hipError_t launch_scan_i32_to_i64(const int32_t *in, int64_t n, int64_t *out, int64_t *block_tmp,
                                  unsigned long long *total_out, hipStream_t s);
int64_t scan_tmp_elems(int64_t n);
hipError_t launch_fill_i32(int32_t *p, int64_t n, int32_t v, hipStream_t s);
hipError_t launch_fill_u64(unsigned long long *p, int64_t n, unsigned long long v, hipStream_t s);
hipError_t launch_count_overflow(int64_t m, const int32_t *row_nnz, unsigned long long *count, hipStream_t s);
hipError_t launch_bin_work(int64_t m, const uint8_t *bin_of_row, const int64_t *prod, const int64_t *a_rp,
                           const int32_t *row_nnz, unsigned long long *sums /*3*OCEAN_MAX_BINS, zero*/, hipStream_t s);
hipError_t launch_final_nnz(int64_t m, const int32_t *nnz1, const int32_t *nnz2, int32_t *out, hipStream_t s);

// symbolic.hip
struct SymLaunch {
    const int32_t *rows;   // row ids of this bin
    int64_t count;
    int bin;
    bool query_bitmap;     // bitmap kernel: read a column's bit before setting it (Section 4.1)
    bool may_overflow;     // tables were sized from a guess (assisted binning): a row whose table fills up
                           // reports -1 instead of a count and probing gives up early
};
hipError_t launch_symbolic_bin(const Csr &A, const Csr &B, const SymLaunch &l, int gb_log2, int32_t *nnz_out,
                               int n_wg, unsigned long long *queue, hipStream_t s);

// order.hip
size_t sort_rows_scratch_bytes(int64_t count);
hipError_t launch_sort_b_rows(const Csr &B, int dtype, int32_t *col_out, void *val_out, int32_t *flags, hipStream_t s);
hipError_t launch_sort_rows_by_products(const int64_t *prod, int32_t *rows, int64_t count, void *scratch, hipStream_t s);

// numeric.hip
struct NumLaunch {
    const int32_t *rows;
    int64_t count;
    int bin;
    const int64_t *out_ptr;   // [m+1]: start of each row's output region; capacity = out_ptr[i+1]-out_ptr[i]
    int32_t *out_col;
    void *out_val;
    int32_t *row_nnz;         // written per row: entries produced, or -1 on overflow
    // scratch of NB_HYBRID / NB_GLOBAL
    void *slab;               // hybrid: n_wg slabs of 32768 values, all zero on entry and on exit
    void *pairs;              // hybrid: n_wg lists of 32768 (key, slot) pairs, scratch
    int32_t *gkeys;           // global: n_wg tables of 2^gbits keys, all EMPTY on entry and on exit
    void *gvals;              // global: n_wg tables of 2^gbits values, all zero on entry and on exit
    int gbits;
    int n_wg;                 // persistent workgroups of the hybrid / global kernels
    unsigned long long *queue; // their shared row counter, zero on entry
    double coef;              // global: table slots per reserved output entry
    const uint32_t *bw;       // dense kernel: window boundary table of B, or null to use the global-table kernel
    int n_win;
    bool query_bitmap;        // dense windows: read a column's presence bit before setting it (Section 4.1)
    bool fine_buckets;        // 512- and 1024-slot bins: order the row through 2048 column buckets (clustered columns)
    const int32_t *cmin;      // dense-range bin: first column each row can reach
};
hipError_t launch_window_table(const Csr &B, int dtype, uint32_t *bw, int *n_win_out, int32_t *flags, hipStream_t s);
int heavy_workgroups_per_cu();   // workgroups of the column-window kernel that one compute unit holds
int dense_window_count(int64_t n_cols, int dtype);
hipError_t launch_numeric_bin(const Csr &A, const Csr &B, int dtype, const NumLaunch &l, int gb_log2, hipStream_t s);

// esc.hip
struct EscLaunch {
    const int32_t *rows;      // row ids, each with at most `lanes` intermediate products
    int64_t count;
    int lanes;                // 16 or 32 lanes (= products) per row
    const int64_t *out_ptr;
    int32_t *out_col;
    void *out_val;
    int32_t *row_nnz;
};
constexpr int64_t ESC_MAX_COLS = (1ll << 26) - 1;   // column id and lane number share one 32-bit sort key
hipError_t launch_numeric_esc(const Csr &A, const Csr &B, int dtype, const EscLaunch &l, hipStream_t s);

// compact.hip
hipError_t launch_compact(int64_t m, int dtype, const int64_t *c_rp, const int32_t *nnz1, const int64_t *ptr1,
                          const int32_t *col1, const void *val1, const int64_t *ptr2, const int32_t *col2,
                          const void *val2, int32_t *c_col, void *c_val, int g_log2, int64_t nnz_c, hipStream_t s);

hipError_t launch_compact_range(int64_t m, int dtype, const int64_t *c_rp, const int32_t *nnz1, const int64_t *ptr1,
                                const int32_t *col1, const void *val1, const int64_t *ptr2, const int32_t *col2,
                                const void *val2, int32_t *dst_col, void *dst_val, int64_t first, int64_t last,
                                int64_t dst_off, hipStream_t s);

}  // namespace ocean
