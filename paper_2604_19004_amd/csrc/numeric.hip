// Numeric pass: Gustavson's row-wise product (paper Section 2.1) with
// open-addressing hash accumulators (Section 2.2) sized per bin, followed by
// the per-row sort that makes the output CSR-compliant (Section 4.2).
//
//   k_numeric_group   four short rows per wave (16 lanes per row), 64-slot tables in LDS
//   k_numeric_wave    one wave per row, 256-slot table in LDS
//   k_numeric_wg      one workgroup per row, keys + values + sort buffer in LDS (512..8192 slots)
//   k_numeric_hybrid  32768 keys in LDS, values accumulated in a global slab (Section 3.3,
//                     enhanced hash accumulator); rows leave sorted through an LDS bitmap rank
//   k_numeric_dense   rows beyond any LDS hash table: dense accumulator + bitmap in LDS over
//                     windows of columns (Section 2.2 dense accumulator, iterated over the row's
//                     column range as in Section 3.2); needs B's rows sorted
//   k_numeric_global  whole table in global memory: the fallback when B's rows are unsorted
//
// A row reports overflow (row_nnz = -1) when its table fills up or when it
// produced more entries than the space reserved for it; such rows are redone
// by the caller with bound-sized tables (Section 3.2, overflow handling).
#include "ocean_internal.hpp"
#include "traverse.hpp"

namespace ocean {

template <typename V>
__device__ __forceinline__ void lds_add(V *p, V v)
{
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

template <typename V>
__device__ __forceinline__ void l2_add(V *p, V v)
{
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Find the slot of `key` in an LDS table of 2^BITS slots, inserting it when
// absent.  Linear probing; -1 when the table is full.
template <int BITS>
__device__ __forceinline__ int lds_find_or_insert(int32_t *keys, int32_t key)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    uint32_t h = table_hash(key, BITS);
    for (uint32_t probe = 0; probe <= MASK; ++probe) {
        const int32_t cur = __hip_atomic_load(&keys[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (cur == key) return (int)h;
        if (cur == EMPTY_KEY) {
            const int32_t old = atomicCAS(&keys[h], EMPTY_KEY, key);
            if (old == EMPTY_KEY || old == key) return (int)h;
        }
        h = (h + 1u) & MASK;
    }
    return -1;
}

// Slot of a key known to be present.
template <int BITS>
__device__ __forceinline__ int lds_find(const int32_t *keys, int32_t key)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    uint32_t h = table_hash(key, BITS);
    for (uint32_t probe = 0; probe <= MASK; ++probe) {
        if (keys[h] == key) return (int)h;
        h = (h + 1u) & MASK;
    }
    return 0;
}

__device__ __forceinline__ int pow2_ceil_i32(int x)
{
    return x <= 1 ? 1 : 1 << (32 - __clz(x - 1));
}

// ======================================================== group kernel ====
// G lanes per row, 256/G rows per workgroup, no workgroup barrier anywhere:
// the lanes of a row are part of one wave.
template <typename V, int G, int BITS>
__global__ void __launch_bounds__(256)
k_numeric_group(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
                const int32_t *__restrict__ rows, int64_t count, int gb_log2,
                const int64_t *__restrict__ out_ptr, int32_t *__restrict__ out_col, V *__restrict__ out_val,
                int32_t *__restrict__ row_nnz)
{
    constexpr int SLOTS = 1 << BITS;
    constexpr int R = 256 / G;
    __shared__ int32_t s_keys[R * SLOTS];
    __shared__ int32_t s_sort[R * SLOTS];
    __shared__ V s_vals[R * SLOTS];
    const int rl = threadIdx.x / G;
    const int sub = threadIdx.x % G;
    int32_t *keys = s_keys + rl * SLOTS;
    int32_t *sbuf = s_sort + rl * SLOTS;
    V *vals = s_vals + rl * SLOTS;
    const int gb = 1 << gb_log2;  // lanes that share one row of B (<= G)
    const int sub_b = sub & (gb - 1);
    const int part = sub >> gb_log2;
    const int parts = G >> gb_log2;
    const int group_shift = (lane_id() / G) * G;
    const unsigned long long group_mask = (G == 64) ? ~0ull : ((1ull << G) - 1ull);

    const int64_t r = (int64_t)blockIdx.x * R + rl;
    const bool live = r < count;
    const int64_t row = live ? rows[r] : 0;

    for (int s = sub; s < SLOTS; s += G) { keys[s] = EMPTY_KEY; vals[s] = (V)0; }
    wave_sync();

    bool ovf = false;
    if (live) {
        const int64_t e1 = a_rp[row + 1];
        for (int64_t e = a_rp[row] + part; e < e1; e += parts) {
            const int64_t k = a_col[e];
            const V a = a_val[e];
            const int64_t p1 = b_rp[k + 1];
            for (int64_t p = b_rp[k] + sub_b; p < p1; p += gb) {
                const int32_t j = b_col[p];
                const V v = a * b_val[p];
                const int slot = lds_find_or_insert<BITS>(keys, j);
                if (slot >= 0) lds_add(&vals[slot], v);
                else ovf = true;
            }
        }
    }
    wave_sync();

    // gather the occupied keys of this row's table
    int c = 0;
#pragma unroll
    for (int it = 0; it < SLOTS / G; ++it) {
        const int32_t key = keys[it * G + sub];
        const bool occ = key != EMPTY_KEY;
        const unsigned long long m = (__ballot(occ) >> group_shift) & group_mask;
        if (occ) sbuf[c + __popcll(m & ((1ull << sub) - 1ull))] = key;
        c += __popcll(m);
    }
    const bool ovf_any = ((__ballot(ovf) >> group_shift) & group_mask) != 0;
    const int N = pow2_ceil_i32(c);
    for (int s = c + sub; s < N; s += G) sbuf[s] = SORT_PAD;
    wave_sync();

    // bitonic sort of N keys by the G lanes of the row
    for (int k = 2; k <= N; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = sub; i < (N >> 1); i += G) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int hi = lo | j;
                const int32_t x = sbuf[lo], y = sbuf[hi];
                if ((x > y) == ((lo & k) == 0)) { sbuf[lo] = y; sbuf[hi] = x; }
            }
            wave_sync();
        }
    }

    if (live) {
        const int64_t o = out_ptr[row];
        const int64_t cap = out_ptr[row + 1] - o;
        if (ovf_any || (int64_t)c > cap) {
            if (sub == 0) row_nnz[row] = -1;
        } else {
            for (int t = sub; t < c; t += G) {
                const int32_t key = sbuf[t];
                out_col[o + t] = key;
                out_val[o + t] = vals[lds_find<BITS>(keys, key)];
            }
            if (sub == 0) row_nnz[row] = c;
        }
    }
}

// ========================================================= wave kernel ====
// One wave per row, four rows per workgroup, 256-slot table; entries of the
// row of A are classified by the length of the row of B they reference.
template <typename V>
__global__ void __launch_bounds__(256)
k_numeric_wave(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
               const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
               const int32_t *__restrict__ rows, int64_t count, const int64_t *__restrict__ out_ptr,
               int32_t *__restrict__ out_col, V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int BITS = 8;
    constexpr int SLOTS = 1 << BITS;
    constexpr int R = 4;
    __shared__ int32_t s_keys[R * SLOTS];
    __shared__ int32_t s_sort[R * SLOTS];
    __shared__ V s_vals[R * SLOTS];
    __shared__ WaveQueue<V> s_q[R];
    const int rl = threadIdx.x / WAVE;
    const int sub = lane_id();
    int32_t *keys = s_keys + rl * SLOTS;
    int32_t *sbuf = s_sort + rl * SLOTS;
    V *vals = s_vals + rl * SLOTS;
    const int64_t r = (int64_t)blockIdx.x * R + rl;
    if (r >= count) return;   // whole wave leaves; no workgroup barrier is used below
    const int64_t row = rows[r];
    for (int s = sub; s < SLOTS; s += WAVE) { keys[s] = EMPTY_KEY; vals[s] = (V)0; }
    wave_sync();
    bool ovf = false;
    wave_traverse<true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                        [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                        b_col, b_val, s_q[rl], [&](int32_t j, V v) {
                            const int slot = lds_find_or_insert<BITS>(keys, j);
                            if (slot >= 0) lds_add(&vals[slot], v);
                            else ovf = true;
                        });
    wave_sync();
    int c = 0;
#pragma unroll
    for (int it = 0; it < SLOTS / WAVE; ++it) {
        const int32_t key = keys[it * WAVE + sub];
        const bool occ = key != EMPTY_KEY;
        const unsigned long long m = __ballot(occ);
        if (occ) sbuf[c + __popcll(m & ((1ull << sub) - 1ull))] = key;
        c += __popcll(m);
    }
    const bool ovf_any = __ballot(ovf) != 0;
    const int N = pow2_ceil_i32(c);
    for (int s = c + sub; s < N; s += WAVE) sbuf[s] = SORT_PAD;
    wave_sync();
    for (int k = 2; k <= N; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = sub; i < (N >> 1); i += WAVE) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int hi = lo | j;
                const int32_t x = sbuf[lo], y = sbuf[hi];
                if ((x > y) == ((lo & k) == 0)) { sbuf[lo] = y; sbuf[hi] = x; }
            }
            wave_sync();
        }
    }
    const int64_t o = out_ptr[row];
    const int64_t cap = out_ptr[row + 1] - o;
    if (ovf_any || (int64_t)c > cap) {
        if (sub == 0) row_nnz[row] = -1;
    } else {
        for (int t = sub; t < c; t += WAVE) {
            const int32_t key = sbuf[t];
            out_col[o + t] = key;
            out_val[o + t] = vals[lds_find<BITS>(keys, key)];
        }
        if (sub == 0) row_nnz[row] = c;
    }
}

// =================================================== workgroup helpers ====
template <int THREADS>
__device__ __forceinline__ int block_exclusive_scan_i32(int v, int *s_wave, int &total)
{
    int inc = v;
    for (int off = 1; off < WAVE; off <<= 1) {
        const int o = __shfl_up(inc, off, WAVE);
        if (lane_id() >= off) inc += o;
    }
    const int w = threadIdx.x / WAVE;
    if (lane_id() == WAVE - 1) s_wave[w] = inc;
    __syncthreads();
    int wave_off = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < THREADS / WAVE; ++i) {
        const int x = s_wave[i];
        if (i < w) wave_off += x;
        tot += x;
    }
    __syncthreads();
    total = tot;
    return wave_off + inc - v;
}

// ==================================================== workgroup kernel ====
template <typename V, int BITS, int THREADS>
__global__ void __launch_bounds__(THREADS)
k_numeric_wg(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
             const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
             const int32_t *__restrict__ rows, int64_t count, const int64_t *__restrict__ out_ptr,
             int32_t *__restrict__ out_col, V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int SLOTS = 1 << BITS;
    constexpr int PER = SLOTS / THREADS;
    __shared__ int32_t s_keys[SLOTS];
    __shared__ int32_t s_sort[SLOTS];
    __shared__ V s_vals[SLOTS];
    __shared__ TravQueue<V, THREADS> s_q;
    __shared__ int s_wave[THREADS / WAVE];
    __shared__ int s_ovf;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (r >= count) return;
    const int64_t row = rows[r];

    for (int s = tid; s < SLOTS; s += THREADS) { s_keys[s] = EMPTY_KEY; s_vals[s] = (V)0; }
    if (tid == 0) { s_ovf = 0; s_q.n = 0; s_q.n_huge = 0; }
    __syncthreads();

    TravState ts;
    wg_traverse<THREADS, true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                               [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                               b_col, b_val, s_q, ts, [&](int32_t j, V v) {
                                   const int slot = lds_find_or_insert<BITS>(s_keys, j);
                                   if (slot >= 0) lds_add(&s_vals[slot], v);
                                   else s_ovf = 1;
                               });
    // wg_traverse ends with a barrier (or did nothing for an empty row)
    __syncthreads();

    // compaction of the keys: each thread owns PER consecutive slots
    int mine = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) mine += (s_keys[tid * PER + q] != EMPTY_KEY);
    int c;
    int pos = block_exclusive_scan_i32<THREADS>(mine, s_wave, c);
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int32_t key = s_keys[tid * PER + q];
        if (key != EMPTY_KEY) s_sort[pos++] = key;
    }
    const int N = pow2_ceil_i32(c);
    for (int s = c + tid; s < N; s += THREADS) s_sort[s] = SORT_PAD;
    __syncthreads();

    for (int k = 2; k <= N; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < (N >> 1); i += THREADS) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int hi = lo | j;
                const int32_t x = s_sort[lo], y = s_sort[hi];
                if ((x > y) == ((lo & k) == 0)) { s_sort[lo] = y; s_sort[hi] = x; }
            }
            __syncthreads();
        }
    }

    const int64_t o = out_ptr[row];
    const int64_t cap = out_ptr[row + 1] - o;
    if (s_ovf || (int64_t)c > cap) {
        if (tid == 0) row_nnz[row] = -1;
    } else {
        for (int t = tid; t < c; t += THREADS) {
            const int32_t key = s_sort[t];
            out_col[o + t] = key;
            out_val[o + t] = s_vals[lds_find<BITS>(s_keys, key)];
        }
        if (tid == 0) row_nnz[row] = c;
    }
}

// ======================================================= hybrid kernel ====
// Keys of a 32768-slot table stay in LDS; values are accumulated with
// fire-and-forget atomics into this workgroup's slab in global memory (it is
// 256 KB, so it lives in the L2 of the XCD the workgroup runs on).  The row is
// emitted in ascending order without a comparison sort: the (key, slot) pairs
// are first dumped to a list in global memory, which frees the 128 KB of keys
// for a bitmap over 512 K columns plus its per-word prefix popcount; a key's
// rank in the row is then the number of set bits below it.
constexpr int HY_BITS = 15;
constexpr int HY_SLOTS = 1 << HY_BITS;
constexpr int HY_THREADS = 1024;
constexpr int HY_WIN = 524288;          // columns per ranking window
constexpr int HY_WORDS = HY_WIN / 32;   // 16384 bitmap words + 16384 prefix words = the key table's 128 KB
constexpr int HY_QCAP = 1024;

template <typename V>
__global__ void __launch_bounds__(HY_THREADS)
k_numeric_hybrid(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                 const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
                 const int32_t *__restrict__ rows, int64_t count, unsigned long long *queue,
                 V *__restrict__ slab_all, uint2 *__restrict__ pairs_all, const int64_t *__restrict__ out_ptr,
                 int32_t *__restrict__ out_col, V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int PER = HY_SLOTS / HY_THREADS;   // 32 slots per thread
    constexpr int WPT = HY_WORDS / HY_THREADS;   // 16 bitmap words per thread
    __shared__ int32_t s_keys[HY_SLOTS];
    __shared__ TravQueue<V, HY_QCAP> s_q;
    __shared__ int s_wave[HY_THREADS / WAVE];
    __shared__ int s_ovf;
    __shared__ int s_min, s_max;
    __shared__ unsigned int s_cnt;
    __shared__ long long s_row;
    uint32_t *s_bm = reinterpret_cast<uint32_t *>(s_keys);   // valid only after the keys were dumped
    uint32_t *s_pre = s_bm + HY_WORDS;
    const int tid = threadIdx.x;
    V *slab = slab_all + (size_t)blockIdx.x * HY_SLOTS;
    uint2 *pairs = pairs_all + (size_t)blockIdx.x * HY_SLOTS;

    for (;;) {
        if (tid == 0) s_row = (long long)atomicAdd(queue, 1ull);
        __syncthreads();
        const int64_t r = s_row;
        if (r >= count) break;   // uniform: every wave of the workgroup leaves here
        const int64_t row = rows[r];
        for (int s = tid; s < HY_SLOTS; s += HY_THREADS) s_keys[s] = EMPTY_KEY;
        if (tid == 0) { s_ovf = 0; s_min = 0x7fffffff; s_max = -1; s_cnt = 0; s_q.n = 0; s_q.n_huge = 0; }
        __syncthreads();

        TravState ts;
        wg_traverse<HY_THREADS, true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                                      [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                      b_col, b_val, s_q, ts, [&](int32_t j, V v) {
                                          const int slot = lds_find_or_insert<HY_BITS>(s_keys, j);
                                          if (slot >= 0) l2_add(&slab[slot], v);
                                          else s_ovf = 1;
                                      });
        __threadfence();   // the slab additions are in L2 before anyone exchanges them out
        __syncthreads();

        // dump (key, slot) pairs; one LDS atomic per wave and pass
        int kmin = 0x7fffffff, kmax = -1;
        for (int q = 0; q < PER; ++q) {
            const int slot = q * HY_THREADS + tid;
            const int32_t key = s_keys[slot];
            const bool occ = key != EMPTY_KEY;
            const unsigned long long m = __ballot(occ);
            unsigned int base = 0;
            if (lane_id() == 0 && m) base = atomicAdd(&s_cnt, (unsigned int)__popcll(m));
            base = __shfl(base, 0, WAVE);
            if (occ) {
                pairs[base + __popcll(m & ((1ull << lane_id()) - 1ull))] = make_uint2((unsigned)key, (unsigned)slot);
                kmin = key < kmin ? key : kmin;
                kmax = key > kmax ? key : kmax;
            }
        }
        kmin = -group_reduce_max(-kmin, WAVE);
        kmax = group_reduce_max(kmax, WAVE);
        if (lane_id() == 0) { atomicMin(&s_min, kmin); atomicMax(&s_max, kmax); }
        __threadfence();   // the pairs are read back by other waves of this workgroup
        __syncthreads();

        const int64_t o = out_ptr[row];
        const int64_t cap = out_ptr[row + 1] - o;
        const int lo_key = s_min, hi_key = s_max;
        const int c = (int)s_cnt;
        int done = 0;
        for (int64_t w0 = (int64_t)(lo_key >= 0 ? lo_key : 0) & ~(int64_t)(HY_WIN - 1); w0 <= (int64_t)hi_key; w0 += HY_WIN) {
#pragma unroll
            for (int q = 0; q < WPT; ++q) s_bm[q * HY_THREADS + tid] = 0u;
            __syncthreads();
            for (int i = tid; i < c; i += HY_THREADS) {
                const int64_t d = (int64_t)(int32_t)__hip_atomic_load(&pairs[i].x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - w0;
                if (d >= 0 && d < HY_WIN) atomicOr(&s_bm[d >> 5], 1u << (d & 31));
            }
            __syncthreads();
            int cnt[WPT];
            int mine = 0;
#pragma unroll
            for (int q = 0; q < WPT; ++q) { cnt[q] = __popc(s_bm[tid * WPT + q]); mine += cnt[q]; }
            int wtotal;
            int run = block_exclusive_scan_i32<HY_THREADS>(mine, s_wave, wtotal);
#pragma unroll
            for (int q = 0; q < WPT; ++q) { s_pre[tid * WPT + q] = (uint32_t)run; run += cnt[q]; }
            __syncthreads();
            for (int i = tid; i < c; i += HY_THREADS) {
                const int32_t key = (int32_t)__hip_atomic_load(&pairs[i].x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int64_t d = (int64_t)key - w0;
                if (d >= 0 && d < HY_WIN) {
                    const int slot = (int)__hip_atomic_load(&pairs[i].y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const int rank = done + (int)s_pre[d >> 5] + __popc(s_bm[d >> 5] & ((1u << (d & 31)) - 1u));
                    const V val = __hip_atomic_exchange(&slab[slot], (V)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((int64_t)rank < cap) { out_col[o + rank] = key; out_val[o + rank] = val; }
                }
            }
            done += wtotal;
            __syncthreads();
        }
        if (tid == 0) row_nnz[row] = (s_ovf || (int64_t)done > cap) ? -1 : done;
        __threadfence();
        __syncthreads();
    }
}

// ======================================================== dense kernel ====
// Rows whose output exceeds every hash table.  The column range is cut into
// windows of WIN columns; for one window the workgroup holds a dense array of
// WIN values plus a presence bitmap in LDS, adds every product that falls into
// the window (one LDS add + one LDS or, both without return), then walks the
// bitmap: its prefix popcount places each present column directly at its
// sorted position in the row's output.  bw[k*(n_win+1)+w] is the position in
// B's arrays of the first entry of row k with column >= w*WIN (rows of B must
// be sorted), so a window only visits its own products.  One workgroup takes
// the windows of a row in turn, carrying the running output offset.
constexpr int DN_THREADS = 1024;

template <typename V>
struct DenseCfg {
    static constexpr int WIN = 131072 / (int)sizeof(V);   // 16384 columns (fp64), 32768 (fp32): 128 KB of values
    static constexpr int WORDS = WIN / 32;
};

template <typename V>
__global__ void __launch_bounds__(DN_THREADS)
k_numeric_dense(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                const uint32_t *__restrict__ bw, int n_win, const int32_t *__restrict__ b_col,
                const V *__restrict__ b_val, const int32_t *__restrict__ rows, int64_t count,
                unsigned long long *queue, const int64_t *__restrict__ out_ptr, int32_t *__restrict__ out_col,
                V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int WIN = DenseCfg<V>::WIN;
    constexpr int WORDS = DenseCfg<V>::WORDS;
    __shared__ V s_vals[WIN];
    __shared__ uint32_t s_bm[WORDS];
    __shared__ uint32_t s_pre[WORDS];
    __shared__ TravQueue<V, DN_THREADS> s_q;
    __shared__ int s_wave[DN_THREADS / WAVE];
    __shared__ long long s_row;
    const int tid = threadIdx.x;
    for (int j = tid; j < WIN; j += DN_THREADS) s_vals[j] = (V)0;
    for (int j = tid; j < WORDS; j += DN_THREADS) s_bm[j] = 0u;
    const size_t stride = (size_t)n_win + 1;

    for (;;) {
        if (tid == 0) { s_row = (long long)atomicAdd(queue, 1ull); s_q.n = 0; s_q.n_huge = 0; }
        __syncthreads();
        const int64_t r = s_row;
        if (r >= count) break;   // uniform exit
        const int64_t row = rows[r];
        const int64_t e0 = a_rp[row], e1 = a_rp[row + 1];
        const int64_t o = out_ptr[row];
        const int64_t cap = out_ptr[row + 1] - o;
        long long done = 0;
        TravState ts;   // the queue counters were reset with s_row and keep running over the windows of this row
        for (int w = 0; w < n_win; ++w) {
            const uint32_t *bww = bw + w;
            wg_traverse<DN_THREADS, true>(a_col, a_val, e0, e1,
                                          [&](int32_t k, int64_t &p0, int64_t &len) {
                                              const uint32_t *t = bww + (size_t)k * stride;
                                              const uint32_t a0 = t[0], a1 = t[1];
                                              p0 = a0; len = (int64_t)a1 - (int64_t)a0;
                                          },
                                          b_col, b_val, s_q, ts, [&](int32_t j, V v) {
                                              const unsigned d = (unsigned)(j - w * WIN);
                                              if (d < (unsigned)WIN) {   // always true for a consistent window table
                                                  lds_add(&s_vals[d], v);
                                                  atomicOr(&s_bm[d >> 5], 1u << (d & 31));
                                              }
                                          });
            // all adds of this window are done (wg_traverse ends with a barrier)
            const uint32_t word = tid < WORDS ? s_bm[tid] : 0u;
            int wtotal;
            const int ex = block_exclusive_scan_i32<DN_THREADS>(__popc(word), s_wave, wtotal);
            if (tid < WORDS) s_pre[tid] = (uint32_t)ex;
            __syncthreads();
            if (wtotal > 0) {
                // every thread owns BPT consecutive bits of the bitmap and walks only the set ones
                constexpr int BPT = WIN / DN_THREADS;   // 16 (fp64) or 32 (fp32)
                const int32_t col0 = w * WIN;
                const int j0 = tid * BPT;
                const uint32_t wbits = s_bm[j0 >> 5];
                uint32_t bits = BPT == 32 ? wbits : ((wbits >> (j0 & 31)) & ((1u << (BPT & 31)) - 1u));
                long long rank = done + (long long)s_pre[j0 >> 5] + __popc(wbits & ((1u << (j0 & 31)) - 1u));
                while (bits) {
                    const int b = __ffs((int)bits) - 1;
                    bits &= bits - 1u;
                    const int j = j0 + b;
                    const V val = s_vals[j];
                    s_vals[j] = (V)0;
                    if (rank < cap) { out_col[o + rank] = col0 + j; out_val[o + rank] = val; }
                    ++rank;
                }
                __syncthreads();
                if (tid < WORDS) s_bm[tid] = 0u;
                done += wtotal;
            }
            __syncthreads();
        }
        if (tid == 0) row_nnz[row] = done > cap ? -1 : (int32_t)done;
        __syncthreads();
    }
}

// Positions of the column-window boundaries inside every row of B:
// bw[k*(n_win+1)+w] = first position p in row k with col[p] >= w*win (row end if none).
// One 16-lane group per row.  flags |= 8 when a row is not sorted ascending.
__global__ void __launch_bounds__(256)
k_window_table(const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, int64_t rows, int win_log2,
               int n_win, uint32_t *__restrict__ bw, int32_t *flags)
{
    const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t k = gt >> 4;
    const int sub = (int)(gt & 15);
    if (k >= rows) return;
    const int64_t p0 = b_rp[k], p1 = b_rp[k + 1];
    uint32_t *t = bw + (size_t)k * ((size_t)n_win + 1);
    bool unsorted = false;
    if (p0 == p1) {
        for (int w = sub; w <= n_win; w += 16) t[w] = (uint32_t)p0;
        return;
    }
    for (int64_t p = p0 + sub; p < p1; p += 16) {
        const int32_t c = b_col[p];
        const int wc = c >> win_log2;
        int wprev = -1;
        if (p > p0) {
            const int32_t cp = b_col[p - 1];
            unsorted |= cp > c;
            wprev = cp >> win_log2;
        }
        for (int w = wprev + 1; w <= wc; ++w) t[w] = (uint32_t)p;
        if (p == p1 - 1)
            for (int w = wc + 1; w <= n_win; ++w) t[w] = (uint32_t)p1;
    }
    if (unsorted) atomicOr(flags, 8);
}

hipError_t launch_window_table(const Csr &B, int dtype, uint32_t *bw, int *n_win_out, int32_t *flags, hipStream_t s)
{
    const int win_log2 = dtype == OCEAN_F64 ? 14 : 15;
    const int n_win = (int)((B.cols + (1ll << win_log2) - 1) >> win_log2);
    *n_win_out = n_win;
    if (B.rows == 0) return hipSuccess;
    const int64_t threads = B.rows * 16;
    hipLaunchKernelGGL(k_window_table, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, B.rp, B.col, B.rows,
                       win_log2, n_win, bw, flags);
    return hipGetLastError();
}

int dense_window_count(int64_t n_cols, int dtype)
{
    const int win_log2 = dtype == OCEAN_F64 ? 14 : 15;
    return (int)((n_cols + (1ll << win_log2) - 1) >> win_log2);
}

// ======================================================= global kernel ====
// The table of a row lives in this workgroup's region of global memory
// (tables are EMPTY / zero between rows).  Rows are emitted in order through
// an LDS bitmap over windows of 512 K columns, which also restores the table.
constexpr int GL_THREADS = 1024;
constexpr int GL_WIN = 524288;
constexpr int GL_WORDS = GL_WIN / 32;   // 16384
constexpr int GL_QCAP = 1024;

__device__ __forceinline__ int64_t gl_find_or_insert(int32_t *keys, int bits, int32_t key)
{
    const uint32_t mask = (1u << bits) - 1u;
    uint32_t h = table_hash(key, bits);
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const int32_t cur = __hip_atomic_load(&keys[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cur == key) return h;
        if (cur == EMPTY_KEY) {
            const int32_t old = atomicCAS(&keys[h], EMPTY_KEY, key);
            if (old == EMPTY_KEY || old == key) return h;
        }
        h = (h + 1u) & mask;
    }
    return -1;
}

template <typename V>
__global__ void __launch_bounds__(GL_THREADS)
k_numeric_global(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                 const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
                 const int32_t *__restrict__ rows, int64_t count, unsigned long long *queue,
                 int32_t *__restrict__ gkeys_all, V *__restrict__ gvals_all, int gbits_max, double coef,
                 const int64_t *__restrict__ out_ptr, int32_t *__restrict__ out_col, V *__restrict__ out_val,
                 int32_t *__restrict__ row_nnz)
{
    constexpr int WPT = GL_WORDS / GL_THREADS;   // 16 words per thread
    __shared__ uint32_t s_bm[GL_WORDS];
    __shared__ uint32_t s_pre[GL_WORDS];
    __shared__ TravQueue<V, GL_QCAP> s_q;
    __shared__ int s_wave[GL_THREADS / WAVE];
    __shared__ int s_ovf;
    __shared__ int s_min, s_max;
    __shared__ long long s_row;
    const int tid = threadIdx.x;
    int32_t *gk = gkeys_all + ((size_t)blockIdx.x << gbits_max);
    V *gv = gvals_all + ((size_t)blockIdx.x << gbits_max);

    for (;;) {
        if (tid == 0) s_row = (long long)atomicAdd(queue, 1ull);
        __syncthreads();
        const int64_t r = s_row;
        if (r >= count) break;
        const int64_t row = rows[r];
        const int64_t o = out_ptr[row];
        const int64_t cap = out_ptr[row + 1] - o;
        // table size of this row: a power of two holding coef * capacity, at most the region
        int bits = 10;
        {
            const double want = coef * (double)cap;
            while (bits < gbits_max && (double)(1ll << bits) < want) ++bits;
        }
        const int64_t slots = 1ll << bits;
        if (tid == 0) { s_ovf = 0; s_min = 0x7fffffff; s_max = -1; s_q.n = 0; s_q.n_huge = 0; }
        __syncthreads();

        int kmin = 0x7fffffff, kmax = -1;
        TravState ts;
        wg_traverse<GL_THREADS, true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                                      [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                      b_col, b_val, s_q, ts, [&](int32_t j, V v) {
                                          const int64_t slot = gl_find_or_insert(gk, bits, j);
                                          if (slot >= 0) {
                                              l2_add(&gv[slot], v);
                                              kmin = j < kmin ? j : kmin;
                                              kmax = j > kmax ? j : kmax;
                                          } else {
                                              s_ovf = 1;
                                          }
                                      });
        kmin = -group_reduce_max(-kmin, WAVE);
        kmax = group_reduce_max(kmax, WAVE);
        if (lane_id() == 0) { atomicMin(&s_min, kmin); atomicMax(&s_max, kmax); }
        __threadfence();
        __syncthreads();

        const int lo_key = s_min, hi_key = s_max;
        long long done = 0;
        for (int64_t w0 = (int64_t)(lo_key >= 0 ? lo_key : 0) & ~(int64_t)(GL_WIN - 1); w0 <= (int64_t)hi_key; w0 += GL_WIN) {
#pragma unroll
            for (int q = 0; q < WPT; ++q) s_bm[tid * WPT + q] = 0u;
            __syncthreads();
            for (int64_t s = tid; s < slots; s += GL_THREADS) {
                const int32_t key = __hip_atomic_load(&gk[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int64_t d = (int64_t)key - w0;
                if (key != EMPTY_KEY && d >= 0 && d < GL_WIN) atomicOr(&s_bm[d >> 5], 1u << (d & 31));
            }
            __syncthreads();
            int cnt[WPT];
            int mine = 0;
#pragma unroll
            for (int q = 0; q < WPT; ++q) { cnt[q] = __popc(s_bm[tid * WPT + q]); mine += cnt[q]; }
            int wtotal;
            int run = block_exclusive_scan_i32<GL_THREADS>(mine, s_wave, wtotal);
#pragma unroll
            for (int q = 0; q < WPT; ++q) { s_pre[tid * WPT + q] = (uint32_t)run; run += cnt[q]; }
            __syncthreads();
            for (int64_t s = tid; s < slots; s += GL_THREADS) {
                const int32_t key = __hip_atomic_load(&gk[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int64_t d = (int64_t)key - w0;
                if (key != EMPTY_KEY && d >= 0 && d < GL_WIN) {
                    const long long rank = done + (long long)s_pre[d >> 5] + __popc(s_bm[d >> 5] & ((1u << (d & 31)) - 1u));
                    const V val = __hip_atomic_exchange(&gv[s], (V)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(&gk[s], EMPTY_KEY, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (rank < cap) { out_col[o + rank] = key; out_val[o + rank] = val; }
                }
            }
            done += wtotal;
            __syncthreads();
        }
        if (tid == 0) row_nnz[row] = (s_ovf || done > cap) ? -1 : (int32_t)done;
        __threadfence();
        __syncthreads();
    }
}

// ============================================================ dispatch ====
template <typename V>
static hipError_t dispatch(const Csr &A, const Csr &B, const NumLaunch &l, int gb_log2, hipStream_t s)
{
    if (l.count <= 0) return hipSuccess;
    const V *av = static_cast<const V *>(A.val);
    const V *bv = static_cast<const V *>(B.val);
    V *ov = static_cast<V *>(l.out_val);
#define OCEAN_WG(BITS, THREADS)                                                                                   \
    hipLaunchKernelGGL((k_numeric_wg<V, BITS, THREADS>), dim3((unsigned)l.count), dim3(THREADS), 0, s, A.rp, A.col, \
                       av, B.rp, B.col, bv, l.rows, l.count, l.out_ptr, l.out_col, ov, l.row_nnz)
    switch (l.bin) {
    case NB_G16: {
        const int64_t blocks = (l.count + 15) / 16;
        hipLaunchKernelGGL((k_numeric_group<V, 16, 6>), dim3((unsigned)blocks), dim3(256), 0, s, A.rp, A.col, av, B.rp,
                           B.col, bv, l.rows, l.count, gb_log2 < 4 ? gb_log2 : 4, l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    }
    case NB_W64: {
        const int64_t blocks = (l.count + 3) / 4;
        hipLaunchKernelGGL((k_numeric_wave<V>), dim3((unsigned)blocks), dim3(256), 0, s, A.rp, A.col, av, B.rp, B.col, bv,
                           l.rows, l.count, l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    }
    case NB_S512: OCEAN_WG(9, 128); break;
    case NB_S1K: OCEAN_WG(10, 256); break;
    case NB_S2K: OCEAN_WG(11, 512); break;
    case NB_S4K: OCEAN_WG(12, 1024); break;
    case NB_S8K: OCEAN_WG(13, 1024); break;
    case NB_HYBRID:
        hipLaunchKernelGGL((k_numeric_hybrid<V>), dim3((unsigned)l.n_wg), dim3(HY_THREADS), 0, s, A.rp, A.col, av, B.rp,
                           B.col, bv, l.rows, l.count, l.queue, static_cast<V *>(l.slab), static_cast<uint2 *>(l.pairs),
                           l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    case NB_GLOBAL:
        if (l.bw != nullptr)
            hipLaunchKernelGGL((k_numeric_dense<V>), dim3((unsigned)l.n_wg), dim3(DN_THREADS), 0, s, A.rp, A.col, av, l.bw,
                               l.n_win, B.col, bv, l.rows, l.count, l.queue, l.out_ptr, l.out_col, ov, l.row_nnz);
        else
            hipLaunchKernelGGL((k_numeric_global<V>), dim3((unsigned)l.n_wg), dim3(GL_THREADS), 0, s, A.rp, A.col, av,
                               B.rp, B.col, bv, l.rows, l.count, l.queue, l.gkeys, static_cast<V *>(l.gvals), l.gbits,
                               l.coef, l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    default: return hipErrorInvalidValue;
    }
#undef OCEAN_WG
    return hipGetLastError();
}

hipError_t launch_numeric_bin(const Csr &A, const Csr &B, int dtype, const NumLaunch &l, int gb_log2, hipStream_t s)
{
    return dtype == OCEAN_F64 ? dispatch<double>(A, B, l, gb_log2, s) : dispatch<float>(A, B, l, gb_log2, s);
}

}  // namespace ocean
