// Numeric pass: Gustavson's row-wise product (paper Section 2.1) with
// open-addressing hash accumulators (Section 2.2) sized per bin, followed by
// the per-row sort that makes the output CSR-compliant (Section 4.2).
//
//   k_numeric_group   several short rows per wave (8 or 16 lanes per row), 32- or 64-slot tables in LDS
//   k_numeric_wave    one wave per row, 256-slot table in LDS
//   k_numeric_wg      one workgroup per row, keys + values + sort buffer in LDS (512..8192 slots)
//   k_numeric_hybrid  32768 keys in LDS, values accumulated in a global slab (Section 3.3,
//                     enhanced hash accumulator); rows leave sorted through an LDS bitmap rank
//   k_numeric_heavy   rows beyond the 4096-slot table when B's rows are sorted: column windows, each
//                     accumulated in LDS either densely (values + bitmap, Section 2.2 dense
//                     accumulator iterated over the row's column range as in Section 3.2) or, for
//                     sparse stretches of several windows, by staging the products in LDS and
//                     adding them at the bitmap rank of their column (no hash table)
//   k_numeric_global  whole table in global memory, and k_numeric_hybrid: the path of such rows
//                     when B's rows are unsorted (or the window table would be too large)
//
// A row reports overflow (row_nnz = -1) when its table fills up or when it
// produced more entries than the space reserved for it; such rows are redone
// by the caller with bound-sized tables (Section 3.2, overflow handling).
#include "ocean_internal.hpp"
#include "traverse.hpp"

namespace ocean {

// The type values are accumulated in inside LDS.  fp32 products are added up in fp64: the LDS atomic ds_add_f32
// measured about twenty times slower than ds_add_f64 on this GPU (a block-diagonal input, same structure in both
// types: dense accumulation 4.27 ms against 2.40 ms; with plain stores in place of the atomics 1.42 against 2.27 ms),
// so an fp32 row costs the LDS of an fp64 row and is faster for it - and closer to the exact sum.
constexpr int ilog2_const(int x) { return x <= 1 ? 0 : 1 + ilog2_const(x >> 1); }

template <typename V> struct AccOf { using type = V; };
template <> struct AccOf<float> { using type = double; };
template <typename V> using acc_t = typename AccOf<V>::type;

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

// Slot of a key known to be present.
template <int BITS>
__device__ __forceinline__ int lds_find(const int32_t *keys, int32_t key)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    uint32_t h = table_hash(key, BITS);
    const uint32_t step = table_step(key, BITS);
    for (uint32_t probe = 0; probe <= MASK; ++probe) {
        if (keys[h] == key) return (int)h;
        h = (h + step) & MASK;
    }
    return 0;
}

// Add a batch of products to an LDS hash table (keys / vals of 2^BITS slots).
// A wave waits for its slowest lane, so the cost of inserting is set by the
// longest probe sequence among its lanes, not by the average.  Two measures
// keep that short: probe strides depend on the key (double hashing, no
// clustering), and every lane walks its own U products at its own pace - a
// lane that has placed a product goes on to its next one while other lanes are
// still probing, so the wave-wide loop runs for the largest per-lane SUM of
// probes instead of the sum of per-product maxima.  One compare-and-swap per
// lane and round; the value is added as soon as the slot is known
// (add(slot, value, whether the key is new to the table)).  Valid products come
// first in a batch (cj < 0 ends it).  False when the table is full.
template <int BITS, int U, typename V, typename AddFn>
__device__ __forceinline__ bool lds_insert_batch(int32_t *keys, const int32_t (&cj)[U], const V (&cv)[U], AddFn add)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    int idx = 0;
    int32_t key = cj[0];
    V val = cv[0];
    uint32_t h = table_hash(key, BITS);
    uint32_t step = table_step(key, BITS);
    uint32_t rounds = 0;
    bool ok = true;
    while (key >= 0) {
        const int32_t old = atomicCAS(&keys[h], EMPTY_KEY, key);
        if (old == EMPTY_KEY || old == key) {
            add((int)h, val, old == EMPTY_KEY);
            ++idx;
            key = -1;
#pragma unroll
            for (int u = 1; u < U; ++u)
                if (idx == u) { key = cj[u]; val = cv[u]; }
            h = table_hash(key, BITS);
            step = table_step(key, BITS);
            rounds = 0;
        } else {
            h = (h + step) & MASK;
            if (++rounds > MASK) { ok = false; key = -1; }
        }
    }
    return ok;
}

__device__ __forceinline__ int pow2_ceil_i32(int x)
{
    return x <= 1 ? 1 : 1 << (32 - __clz(x - 1));
}

// ======================================================== group kernel ====
// Several short rows per wave: G lanes per row (16 with 64-slot tables, 8 with
// 32-slot tables), 256/G rows per workgroup; no workgroup barrier anywhere: the
// lanes of a row are part of one wave.  These rows are bound by the latency of
// their chain of dependent loads (row id -> offsets -> entries -> rows of B ->
// products), so what counts is how many rows a CU has in flight.
template <typename V, int G, int BITS>
__global__ void __launch_bounds__(256)
k_numeric_group(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
                const int32_t *__restrict__ rows, int64_t count, const int64_t *__restrict__ out_ptr,
                int32_t *__restrict__ out_col, V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int SLOTS = 1 << BITS;
    constexpr int R = 256 / G;
    __shared__ int32_t s_keys[R * SLOTS];
    using AV = acc_t<V>;
    __shared__ AV s_vals[R * SLOTS];
    // per row: the traversal's chunk and, when the traversal is done, the gathered keys of the row's table with
    // the slot each came from, in the same memory
    struct Gathered {
        int32_t key[SLOTS];
        uint8_t slot[SLOTS];
    };
    union RowScratch {
        FlatChunk<V, G> fc;
        Gathered g;
    };
    __shared__ RowScratch s_rs[R];
    const int rl = threadIdx.x / G;
    const int sub = threadIdx.x % G;
    int32_t *keys = s_keys + rl * SLOTS;
    int32_t *sbuf = s_rs[rl].g.key;
    uint8_t *slot_of = s_rs[rl].g.slot;
    AV *vals = s_vals + rl * SLOTS;
    const int group_shift = (lane_id() / G) * G;
    const unsigned long long group_mask = (1ull << G) - 1ull;

    const int64_t r = (int64_t)blockIdx.x * R + rl;
    const bool live = r < count;
    const int64_t row = live ? rows[r] : 0;

    for (int s = sub; s < SLOTS; s += G) { keys[s] = EMPTY_KEY; vals[s] = (AV)0; }
    wave_sync();

    bool ovf = false;
    const int64_t e0 = live ? a_rp[row] : 0;
    const int64_t e1 = live ? a_rp[row + 1] : 0;
    auto f = [&](const auto &cj, const auto &cv) {
        if (!lds_insert_batch<BITS>(keys, cj, cv, [&](int slot, V v, bool) { lds_add(&vals[slot], (AV)v); })) ovf = true;
    };
    // the rows of a wave advance together: same number of G-entry chunks for all of them
    const int chunks = (int)wave_max_u32((uint32_t)((e1 - e0 + G - 1) / G));   // (uniform)
    for (int ch = 0; ch < chunks; ++ch) {
        const int64_t e = e0 + (int64_t)ch * G + sub;
        int64_t p0 = 0;
        uint32_t len = 0;
        V a = V();
        if (e < e1) {
            const int64_t k = a_col[e];
            a = a_val[e];
            p0 = b_rp[k];
            len = (uint32_t)(b_rp[k + 1] - p0);
        }
        group_flat<G, true>(s_rs[rl].fc, p0, len, a, b_col, b_val, f);
    }
    wave_sync();

    // gather the occupied keys of this row's table, and where their values are
    int c = 0;
#pragma unroll
    for (int it = 0; it < SLOTS / G; ++it) {
        const int32_t key = keys[it * G + sub];
        const bool occ = key != EMPTY_KEY;
        const unsigned long long m = (__ballot(occ) >> group_shift) & group_mask;
        if (occ) {
            const int at = c + __popcll(m & ((1ull << sub) - 1ull));
            sbuf[at] = key;
            slot_of[at] = (uint8_t)(it * G + sub);
        }
        c += __popcll(m);
    }
    const bool ovf_any = ((__ballot(ovf) >> group_shift) & group_mask) != 0;
    wave_sync();

    // Column order without a sort (Section 4.2 sorts key-pointer pairs; a row this short is cheaper to rank):
    // the place of a key is the number of smaller keys in the row.  Every lane ranks the keys t = sub, sub + G, ...
    // of the gathered list against all c of them, one broadcast read per step; the rows of a wave go through
    // the loop together, as many steps as the longest of them has keys.
    constexpr int T = SLOTS / G;
    const int cmax = (int)wave_max_u32((uint32_t)c);   // uniform for the wave
    int32_t mk[T];
    int rank[T];
#pragma unroll
    for (int i = 0; i < T; ++i) {
        const int t = sub + i * G;
        mk[i] = t < c ? sbuf[t] : SORT_PAD;
        rank[i] = 0;
    }
    // (TT: keys per lane that the longest row of the wave needs ranked)
    auto count_smaller = [&](auto tt) {
        constexpr int TT = decltype(tt)::value;
        for (int j = 0; j < cmax; ++j) {
            const int32_t kr = sbuf[j];                   // (j < SLOTS; beyond the row's keys whatever is there)
            const int32_t kj = j < c ? kr : SORT_PAD;     // nothing is smaller than the pad
#pragma unroll
            for (int i = 0; i < TT; ++i) rank[i] += kj < mk[i];
        }
    };
    if (cmax <= G) count_smaller(std::integral_constant<int, 1>{});
    else if (cmax <= 2 * G) count_smaller(std::integral_constant<int, 2>{});
    else count_smaller(std::integral_constant<int, T>{});

    if (live) {
        const int64_t o = out_ptr[row];
        const int64_t cap = out_ptr[row + 1] - o;
        if (ovf_any || (int64_t)c > cap) {
            if (sub == 0) row_nnz[row] = -1;
        } else {
#pragma unroll
            for (int i = 0; i < T; ++i) {
                const int t = sub + i * G;
                if (t < c) {
                    out_col[o + rank[i]] = mk[i];
                    out_val[o + rank[i]] = (V)vals[slot_of[t]];
                }
            }
            if (sub == 0) row_nnz[row] = c;
        }
    }
}

// =================================================== workgroup helpers ====
// s_wave: one word per wave.  With TRAILING_BARRIER = false the caller keeps s_wave untouched until
// a later barrier of its own.
template <int THREADS, bool TRAILING_BARRIER = true>
__device__ __forceinline__ int block_exclusive_scan_i32(int v, int *s_wave, int &total)
{
    const int inc = (int)wave_inclusive_scan_u32((uint32_t)v);
    const int w = threadIdx.x / WAVE;
    if (lane_id() == WAVE - 1) s_wave[w] = inc;
    __syncthreads();
    uint32_t tot;
    const int wave_off = (int)waves_before_u32<THREADS / WAVE>(reinterpret_cast<const uint32_t *>(s_wave), w, tot);
    if (TRAILING_BARRIER) __syncthreads();
    total = (int)tot;
    return wave_off + inc - v;
}

// Who works on one row: a whole workgroup of THREADS threads, or one wave (THREADS = 64) among several
// in a workgroup that each have a row of their own.  The ordered write-out below is written once for both.
struct WorkgroupScope {
    static __device__ __forceinline__ int tid() { return (int)threadIdx.x; }
    static __device__ __forceinline__ void sync() { __syncthreads(); }
    template <int THREADS>
    static __device__ __forceinline__ int exclusive_scan(int v, int *s_wave, int &total)
    {
        return block_exclusive_scan_i32<THREADS>(v, s_wave, total);
    }
};
struct WaveScope {
    static __device__ __forceinline__ int tid() { return lane_id(); }
    static __device__ __forceinline__ void sync() { wave_sync(); }
    template <int THREADS>
    static __device__ __forceinline__ int exclusive_scan(int v, int *, int &total)
    {
        static_assert(THREADS == WAVE, "one wave");
        const int inc = (int)wave_inclusive_scan_u32((uint32_t)v);
        total = (int)wave_read_lane_u32((uint32_t)inc, WAVE - 1);
        return inc - v;
    }
};

// Write the keys of an LDS hash table to the output in increasing column order
// without sorting them.  Every thread holds PER keys of the table in registers
// (EMPTY_KEY = none; key[q] sits in slot q*THREADS + tid).  The keys are counted
// into NB = THREADS*PER buckets of W = 2^shift columns starting at kmin (all keys
// lie in [kmin, kmin + NB*W)), and a prefix sum over the counts gives every
// bucket its range [start, start + count) of the output, which is also its
// private range of the NB-word array `grouped`.  Inside a bucket the rank of a
// key is found in one of two ways, whichever is cheap for that bucket:
//   * a bucket with fewer keys than the W/32 words of a bitmap over its columns
//     lists its keys in its range (the atomic that counted a key also returned
//     its arrival index) and a key counts the smaller ones among them;
//   * a bucket with at least that many keys (a cluster of columns) has room in
//     its range for that bitmap: the keys set their bits and a key's rank is the
//     number of set bits below its own.
// So clustered and scattered columns cost about the same, a few LDS accesses
// per key.  With BF > 1 there are BF buckets per table slot (NB = THREADS*PER*BF): a
// cluster's bitmap then has fewer words below a key's own, and the threads of a wave
// wait for the longest such count among them.  hist: NB/2 + 1 words, zeroed, two
// 16-bit counts per word.  Returns
// the number of keys; with CHECK, -1 (and nothing written) when some listed
// bucket holds more than `limit` keys, for the caller to sort instead.
// Barriers inside; ends without one.  The table's values are overwritten (the
// keys and values are put in order inside LDS and copied out from there).
// `grouped` may be the table's own key array, provided every thread has read
// its keys before the call (barrier).
template <int THREADS, int PER, bool CHECK, typename Scope = WorkgroupScope, int BF = 1, typename AV, typename V>
__device__ __forceinline__ int bucket_emit(const int32_t (&key)[PER], AV *s_vals, int32_t kmin, int shift,
                                           uint32_t *hist, int32_t *grouped, int *s_wave, int *s_flag, int limit,
                                           int64_t o, int64_t cap, long long done, int32_t *__restrict__ out_col,
                                           V *__restrict__ out_val)
{
    static_assert(PER % 2 == 0, "two buckets per word");
    constexpr int NB = THREADS * PER * BF;   // BF buckets per table slot: narrower buckets, shorter bitmaps to rank in
    constexpr int OWNW = PER * BF / 2;       // words of counts (two buckets each) that a thread owns
    const int tid = Scope::tid();
    const int words = shift > 5 ? 1 << (shift - 5) : 1;   // bitmap words of one bucket
    const uint32_t wmask = (1u << shift) - 1u;
    int arrival[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        arrival[q] = 0;
        if (key[q] != EMPTY_KEY) {
            const uint32_t b = (uint32_t)(key[q] - kmin) >> shift;
            const uint32_t old = atomicAdd(&hist[b >> 1], 1u << ((b & 1u) * 16));
            arrival[q] = (int)((old >> ((b & 1u) * 16)) & 0xffffu);
        }
    }
    Scope::sync();
#pragma unroll
    for (int q = 0; q < PER; ++q) grouped[q * THREADS + tid] = 0;
    // counts -> starts, in place; this thread owns buckets 2*tid*OWNW .. 2*(tid+1)*OWNW - 1
    uint32_t wv[OWNW];
    int sum = 0, kmax = 0;
#pragma unroll
    for (int j = 0; j < OWNW; ++j) {
        wv[j] = hist[tid * OWNW + j];
        const int c0 = (int)(wv[j] & 0xffffu), c1 = (int)(wv[j] >> 16);
        sum += c0 + c1;
        if (c0 < words) kmax = max(kmax, c0);
        if (c1 < words) kmax = max(kmax, c1);
    }
    if (CHECK && kmax > limit) *s_flag = 1;
    int total;
    int base = Scope::template exclusive_scan<THREADS>(sum, s_wave, total);
#pragma unroll
    for (int j = 0; j < OWNW; ++j) {
        const int c0 = (int)(wv[j] & 0xffffu), c1 = (int)(wv[j] >> 16);
        hist[tid * OWNW + j] = (uint32_t)base | ((uint32_t)(base + c0) << 16);
        base += c0 + c1;
    }
    if (tid == THREADS - 1) hist[NB / 2] = (uint32_t)total;
    Scope::sync();
    if (CHECK && *s_flag) return -1;   // uniform
    auto start_of = [&](uint32_t b) { return (int)((hist[b >> 1] >> ((b & 1u) * 16)) & 0xffffu); };
    int lo[PER];
    bool bitmap[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        lo[q] = 0; bitmap[q] = false;
        if (key[q] != EMPTY_KEY) {
            const uint32_t x = (uint32_t)(key[q] - kmin);
            const uint32_t b = x >> shift, d = x & wmask;
            lo[q] = start_of(b);
            bitmap[q] = start_of(b + 1) - lo[q] >= words;
            if (bitmap[q]) atomicOr(reinterpret_cast<uint32_t *>(&grouped[lo[q] + (int)(d >> 5)]), 1u << (d & 31u));
            else grouped[lo[q] + arrival[q]] = key[q];
        }
    }
    Scope::sync();
    int rank[PER];
    AV val[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        rank[q] = 0;
        val[q] = AV();
        if (key[q] != EMPTY_KEY) {
            const uint32_t x = (uint32_t)(key[q] - kmin);
            const uint32_t b = x >> shift, d = x & wmask;
            int r = lo[q];
            if (bitmap[q]) {
                const int dw = (int)(d >> 5);
                for (int j = 0; j < dw; ++j) r += __popc((uint32_t)grouped[lo[q] + j]);
                r += __popc((uint32_t)grouped[lo[q] + dw] & ((1u << (d & 31u)) - 1u));
            } else {
                const int hi = start_of(b + 1);
                for (int i = lo[q]; i < hi; ++i) r += grouped[i] < key[q];
            }
            rank[q] = r;
            val[q] = s_vals[q * THREADS + tid];
        }
    }
    Scope::sync();
    // permute keys and values into place inside LDS (every thread holds its own in registers), so
    // that the row leaves with coalesced stores
#pragma unroll
    for (int q = 0; q < PER; ++q)
        if (key[q] != EMPTY_KEY) { grouped[rank[q]] = key[q]; s_vals[rank[q]] = val[q]; }
    Scope::sync();
    const long long room = cap - done;
    const int n_out = (long long)total < room ? total : (room > 0 ? (int)room : 0);
    for (int i = tid; i < n_out; i += THREADS) {
        out_col[o + done + i] = grouped[i];
        out_val[o + done + i] = (V)s_vals[i];
    }
    return total;
}

// ========================================================= wave kernel ====
// One wave per row, R rows per workgroup, a table of 2^BITS slots (256, 512 or 1024) per row.  No
// workgroup barrier anywhere: traversal, insertion and the ordered write-out (column buckets, as in the
// workgroup kernels) are all wave-synchronous, so a row costs one wave's instructions instead of a
// workgroup's, and none of the waiting at barriers.  Rows of these sizes are bound by instruction issue,
// not by memory.
template <typename V, int BITS, int R>
__global__ void __launch_bounds__(WAVE * R)
k_numeric_wave(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
               const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
               const int32_t *__restrict__ rows, int64_t count, const int64_t *__restrict__ out_ptr,
               int32_t *__restrict__ out_col, V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int SLOTS = 1 << BITS;
    constexpr int PER = SLOTS / WAVE;
    constexpr int BF = 1;
    constexpr int NBK = SLOTS * BF;
    // the traversal's chunk and, after it, the bucket counts of the ordered write-out share one buffer per row
    constexpr size_t HIST_BYTES = (NBK / 2 + 1) * sizeof(uint32_t);
    constexpr size_t SCRATCH = sizeof(FlatChunk<V, WAVE>) > HIST_BYTES ? sizeof(FlatChunk<V, WAVE>) : HIST_BYTES;
    using AV = acc_t<V>;
    __shared__ int32_t s_keys[R * SLOTS];
    __shared__ AV s_vals[R * SLOTS];
    __shared__ __align__(16) unsigned char s_scratch[R][(SCRATCH + 15) / 16 * 16];
    __shared__ int s_flag[R];
    const int rl = threadIdx.x / WAVE;
    const int sub = lane_id();
    int32_t *keys = s_keys + rl * SLOTS;
    AV *vals = s_vals + rl * SLOTS;
    FlatChunk<V, WAVE> &fc = *reinterpret_cast<FlatChunk<V, WAVE> *>(s_scratch[rl]);
    uint32_t *hist = reinterpret_cast<uint32_t *>(s_scratch[rl]);
    const int64_t r = (int64_t)blockIdx.x * R + rl;
    if (r >= count) return;   // whole wave leaves; no workgroup barrier is used below
    const int64_t row = rows[r];
    for (int s = sub; s < SLOTS; s += WAVE) { keys[s] = EMPTY_KEY; vals[s] = (AV)0; }
    wave_sync();
    bool ovf = false;
    wave_traverse<true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                        [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                        b_col, b_val, fc, [&](const auto &cj, const auto &cv) {
                            if (!lds_insert_batch<BITS>(keys, cj, cv, [&](int slot, V v, bool) { lds_add(&vals[slot], (AV)v); })) ovf = true;
                        });
    wave_sync();
    // ---- ordered write-out through column buckets
    int32_t key[PER];
    int lmin = 0x7fffffff, lmax = -1;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        key[q] = keys[q * WAVE + sub];
        if (key[q] != EMPTY_KEY) { lmin = min(lmin, key[q]); lmax = max(lmax, key[q]); }
    }
    for (int j = sub; j < NBK / 2 + 1; j += WAVE) hist[j] = 0u;
    // (column ids are not negative: both extremes as maxima of unsigned numbers)
    const int kmax = (int)wave_max_u32((uint32_t)(lmax + 1)) - 1;
    const int kmin = 0x7fffffff - (int)wave_max_u32((uint32_t)(0x7fffffff - lmin));
    const bool ovf_any = __ballot(ovf) != 0;
    if (kmax < 0) {   // uniform: the row has no entries
        if (sub == 0) row_nnz[row] = 0;
        return;
    }
    wave_sync();   // every lane holds its keys in registers (the key array becomes the buckets' memory), counts are zero
    // smallest shift with (kmax - kmin) >> shift < NBK: the bits of the range beyond those of the bucket count
    static_assert((NBK & (NBK - 1)) == 0, "bucket count is a power of two");
    const int range_bits = 32 - __clz((uint32_t)(kmax - kmin) | 1u);
    const int shift = range_bits > ilog2_const(NBK) ? range_bits - ilog2_const(NBK) : 0;
    const int64_t o = out_ptr[row];
    const int64_t cap = out_ptr[row + 1] - o;
    const int c = bucket_emit<WAVE, PER, false, WaveScope, BF>(key, vals, kmin, shift, hist, keys, nullptr, &s_flag[rl], 0, o, cap, 0,
                                                           out_col, out_val);
    if (sub == 0) row_nnz[row] = (ovf_any || (int64_t)c > cap) ? -1 : c;
}

// ==================================================== workgroup kernel ====
// BF: column buckets per table slot of the ordered write-out (see bucket_emit): 1, or more for inputs with
// clustered columns, up to 2048 buckets.
template <typename V, int BITS, int THREADS, int BF>
__global__ void __launch_bounds__(THREADS)
k_numeric_wg(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
             const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
             const int32_t *__restrict__ rows, int64_t count, const int64_t *__restrict__ out_ptr,
             int32_t *__restrict__ out_col, V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int SLOTS = 1 << BITS;
    constexpr int PER = SLOTS / THREADS;
    constexpr int NBK = SLOTS * BF;
    __shared__ int32_t s_keys[SLOTS];
    using AV = acc_t<V>;
    __shared__ int32_t s_sort[SLOTS];
    __shared__ AV s_vals[SLOTS];
    // the traversal's chunk and, after it, the bucket counts of the ordered write-out share one buffer
    constexpr size_t HIST_BYTES = (NBK / 2 + 1) * sizeof(uint32_t);
    constexpr size_t SCRATCH = sizeof(WgChunk<V, THREADS>) > HIST_BYTES ? sizeof(WgChunk<V, THREADS>) : HIST_BYTES;
    __shared__ __align__(16) unsigned char s_scratch[(SCRATCH + 15) / 16 * 16];
    __shared__ int s_wave[THREADS / WAVE];
    __shared__ int s_ovf, s_min, s_max, s_flag;
    WgChunk<V, THREADS> &s_fc = *reinterpret_cast<WgChunk<V, THREADS> *>(s_scratch);
    uint32_t *s_hist = reinterpret_cast<uint32_t *>(s_scratch);
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (r >= count) return;
    const int64_t row = rows[r];

    for (int s = tid; s < SLOTS; s += THREADS) { s_keys[s] = EMPTY_KEY; s_vals[s] = (AV)0; }
    if (tid == 0) { s_ovf = 0; s_min = 0x7fffffff; s_max = -1; s_flag = 0; }
    __syncthreads();

    wg_traverse<THREADS, true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                               [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                               b_col, b_val, s_fc, [&](const auto &cj, const auto &cv) {
                                   if (!lds_insert_batch<BITS>(s_keys, cj, cv, [&](int slot, V v, bool) { lds_add(&s_vals[slot], (AV)v); }))
                                       s_ovf = 1;
                               });
    // wg_traverse ends with a barrier

    const int64_t o = out_ptr[row];
    const int64_t cap = out_ptr[row + 1] - o;
    // ---- ordered write-out through column buckets
    int32_t key[PER];
    int lmin = 0x7fffffff, lmax = -1;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        key[q] = s_keys[q * THREADS + tid];
        if (key[q] != EMPTY_KEY) { lmin = min(lmin, key[q]); lmax = max(lmax, key[q]); }
    }
    for (int j = tid; j < NBK / 2 + 1; j += THREADS) s_hist[j] = 0u;
    // (column ids are not negative: both extremes as maxima of unsigned numbers)
    lmax = (int)wave_max_u32((uint32_t)(lmax + 1)) - 1;
    lmin = 0x7fffffff - (int)wave_max_u32((uint32_t)(0x7fffffff - lmin));
    if (lane_id() == 0 && lmax >= 0) { atomicMin(&s_min, lmin); atomicMax(&s_max, lmax); }
    __syncthreads();
    const int kmin = __builtin_amdgcn_readfirstlane(s_min), kmax = __builtin_amdgcn_readfirstlane(s_max);   // (the same in every thread)
    if (kmax < 0) {   // uniform: the row has no entries
        if (tid == 0) row_nnz[row] = 0;
        return;
    }
    // smallest shift with (kmax - kmin) >> shift < NBK: the bits of the range beyond those of the bucket count
    static_assert((NBK & (NBK - 1)) == 0, "bucket count is a power of two");
    const int range_bits = 32 - __clz((uint32_t)(kmax - kmin) | 1u);
    const int shift = range_bits > ilog2_const(NBK) ? range_bits - ilog2_const(NBK) : 0;
    constexpr bool CHECK = SLOTS >= 4096;   // smaller tables: even one bucket with every key is cheap to rank
    int c = bucket_emit<THREADS, PER, CHECK, WorkgroupScope, BF>(key, s_vals, kmin, shift, s_hist, s_sort, s_wave, &s_flag, 1024, o, cap, 0,
                                             out_col, out_val);
    if (c >= 0) {
        if (tid == 0) row_nnz[row] = (s_ovf || (int64_t)c > cap) ? -1 : c;
        return;
    }

    // ---- columns too clustered for the buckets: compact the keys, sort them (bitonic), look the values up
    int mine = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) mine += (key[q] != EMPTY_KEY);
    int pos = block_exclusive_scan_i32<THREADS>(mine, s_wave, c);
#pragma unroll
    for (int q = 0; q < PER; ++q)
        if (key[q] != EMPTY_KEY) s_sort[pos++] = key[q];
    const int N = pow2_ceil_i32(c);
    __syncthreads();
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

    if (s_ovf || (int64_t)c > cap) {
        if (tid == 0) row_nnz[row] = -1;
    } else {
        for (int t = tid; t < c; t += THREADS) {
            const int32_t k2 = s_sort[t];
            out_col[o + t] = k2;
            out_val[o + t] = (V)s_vals[lds_find<BITS>(s_keys, k2)];
        }
        if (tid == 0) row_nnz[row] = c;
    }
}

// ================================================== dense-range kernel ====
// Dense accumulator (Section 2.2) over the row's own column range, for rows whose range [cmin, cmin + DS_MAX_COLS)
// is no larger than the hash table they would get (Section 3.3, accumulator selection): one value and one presence
// bit per column of the range in LDS, no keys, no probing, and the row leaves in column order by the bitmap's
// prefix popcount.  QUERY: the presence bit is read first and set only when it is clear (Section 4.1).  A product
// outside the range (B's rows not in column order: the range was a guess) makes the row report overflow, like a
// row with more entries than were reserved for it; the caller redoes such rows with hash tables.
constexpr int DS_THREADS = 256;
constexpr int DS_WORDS = (int)DS_MAX_COLS / 32;
template <typename V, bool QUERY>
__global__ void __launch_bounds__(DS_THREADS)
k_numeric_dspan(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
                const int32_t *__restrict__ rows, int64_t count, const int32_t *__restrict__ cmin,
                const int64_t *__restrict__ out_ptr, int32_t *__restrict__ out_col, V *__restrict__ out_val,
                int32_t *__restrict__ row_nnz)
{
    static_assert(DS_WORDS <= DS_THREADS, "one bitmap word per thread in the prefix sum");
    using AV = acc_t<V>;
    __shared__ AV s_vals[DS_MAX_COLS];
    __shared__ uint32_t s_bm[DS_WORDS];
    __shared__ uint32_t s_pre[DS_WORDS];
    __shared__ WgChunk<V, DS_THREADS> s_fc;
    __shared__ int s_wave[DS_THREADS / WAVE];
    __shared__ int s_bad;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (r >= count) return;
    const int64_t row = rows[r];
    const int32_t c0 = cmin[row];
    for (int j = tid; j < (int)DS_MAX_COLS; j += DS_THREADS) s_vals[j] = (AV)0;
    if (tid < DS_WORDS) s_bm[tid] = 0u;
    if (tid == 0) s_bad = 0;
    __syncthreads();
    wg_traverse<DS_THREADS, true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                                  [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                  b_col, b_val, s_fc, [&](const auto &cj, const auto &cv) {
                                      constexpr int U = sizeof(cj) / sizeof(cj[0]);
#pragma unroll
                                      for (int u = 0; u < U; ++u) {
                                          if (cj[u] < 0) continue;
                                          const uint32_t d = (uint32_t)(cj[u] - c0);   // (a column before c0 wraps to a large number)
                                          if (d < (uint32_t)DS_MAX_COLS) {
                                              lds_add(&s_vals[d], (AV)cv[u]);
                                              const uint32_t bit = 1u << (d & 31u);
                                              if (!QUERY || !(s_bm[d >> 5] & bit)) atomicOr(&s_bm[d >> 5], bit);
                                          } else {
                                              s_bad = 1;
                                          }
                                      }
                                  });
    // (wg_traverse ends with a barrier)
    const uint32_t word = tid < DS_WORDS ? s_bm[tid] : 0u;
    int total;
    const int ex = block_exclusive_scan_i32<DS_THREADS>(__popc(word), s_wave, total);
    if (tid < DS_WORDS) s_pre[tid] = (uint32_t)ex;
    __syncthreads();
    const int64_t o = out_ptr[row];
    const int64_t cap = out_ptr[row + 1] - o;
    if (s_bad || (int64_t)total > cap) {   // uniform
        if (tid == 0) row_nnz[row] = -1;
        return;
    }
    // thread t looks at columns t, t + 256, ...: the lanes of a wave read consecutive values and the present ones
    // among them go to consecutive places of the output
    for (int j = tid; j < (int)DS_MAX_COLS; j += DS_THREADS) {
        const uint32_t wbits = s_bm[j >> 5];
        if ((wbits >> (j & 31)) & 1u) {
            const int rank = (int)s_pre[j >> 5] + __popc(wbits & ((1u << (j & 31)) - 1u));
            out_col[o + rank] = c0 + j;
            out_val[o + rank] = (V)s_vals[j];
        }
    }
    if (tid == 0) row_nnz[row] = total;
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
    __shared__ WgChunk<V, HY_THREADS> s_fc;
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
        if (tid == 0) { s_ovf = 0; s_min = 0x7fffffff; s_max = -1; s_cnt = 0; }
        __syncthreads();

        wg_traverse<HY_THREADS, true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                                      [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                      b_col, b_val, s_fc, [&](const auto &cj, const auto &cv) {
                                          if (!lds_insert_batch<HY_BITS>(s_keys, cj, cv, [&](int slot, V v, bool) { l2_add(&slab[slot], v); }))
                                              s_ovf = 1;
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

// ======================================================== heavy kernel ====
// Rows whose output exceeds the 4096-slot LDS table, when B's rows are sorted.
// The column range is cut into windows of WIN columns and
// bw[k*(n_win+1)+w] is the position in B's arrays of the first entry of row k
// with column >= w*WIN, so any run of windows can be visited on its own.  One
// workgroup first counts the row's products per window (an upper bound of the
// entries of that window), then walks the windows in order, carrying the
// running output offset.  Both kinds of pass accumulate in LDS only, need no
// hash table, and leave their entries in column order:
//   * a window with more products than a sparse pass can stage is accumulated
//     densely (Section 2.2 dense accumulator, iterated over the row's column
//     range as in Section 3.2): WIN values + a presence bitmap in LDS, one LDS
//     add + one LDS or per product; the bitmap's prefix popcount places each
//     present column at its sorted position;
//   * consecutive windows whose products fit the staging memory left beside
//     their bitmap (a sparse stretch: up to 8192 products over 10 windows,
//     fewer over more) share one pass in the manner of an
//     expand-sort-compress accumulator whose sort is a bitmap rank: every
//     product is written to LDS at its own number (no atomics) and marks its
//     column in a bitmap over the stretch; the prefix popcount of the bitmap is
//     the position of each column in the output, so a second sweep over the
//     staged products adds each value at its column's rank.  No probing, no
//     compare-and-swap, no divergence.
// More than half of the kernel's time is the gather of B's entries, which runs
// at what the memory system gives for pieces of rows this short; the rest is
// instruction issue of the work every pass repeats (planning, prefix sums,
// barriers), which is why sparse stretches are merged into few passes and why
// every pass spreads its products over the whole workgroup.
constexpr int HV_THREADS = 1024;
constexpr int HV_REGION = 131072;                  // bytes of LDS that hold the accumulator of a pass
constexpr int HV_WG_PER_CU = 1;                    // (two workgroups of half the size each measured 13 % slower)
constexpr int HV_PPT = 8;                          // products of a sparse pass per thread, at most
constexpr int HV_HCAP = HV_PPT * HV_THREADS;       // products one sparse pass takes at most: 8192
constexpr int HV_MAXWIN = 512;                     // windows per row the kernel can plan for
constexpr int HV_RPT = 48;                         // chunks of up to 48 products per thread find their entries by rank
                                                   // (most dense windows then do: 96.8 -> 94.9 ms; 4 KB more LDS)

template <typename V>
struct DenseCfg {
    static constexpr int WIN = HV_REGION / (int)sizeof(acc_t<V>);   // columns of a window: a region full of accumulators
    static constexpr int WORDS = WIN / 32;
};

// QUERY: dense windows read a column's presence bit and set it only when it is clear (Section 4.1).
template <typename V, bool QUERY>
__global__ void __launch_bounds__(HV_THREADS)
k_numeric_heavy(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                const uint32_t *__restrict__ bw, int n_win, const int32_t *__restrict__ b_col,
                const V *__restrict__ b_val, const int32_t *__restrict__ rows, int64_t count,
                unsigned long long *queue, const int64_t *__restrict__ out_ptr, int32_t *__restrict__ out_col,
                V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int WIN = DenseCfg<V>::WIN;
    constexpr int WORDS = DenseCfg<V>::WORDS;
    // one 128 KB region, used either as the dense window or as hash table + bucket counts
    __shared__ __align__(16) unsigned char s_u[HV_REGION];
    __shared__ uint32_t s_dbm[WORDS];
    __shared__ WgChunk<V, HV_THREADS, HV_RPT> s_fc;
    __shared__ int s_wave[HV_THREADS / WAVE];
    __shared__ uint32_t s_pw[HV_MAXWIN + 1];   // s_pw[w]: products of the row in the windows before w
    __shared__ int s_ovf;
    __shared__ long long s_row;
    static_assert(WORDS <= HV_THREADS, "the prefix counts of a dense window reuse the chunk's array of prefix sums");
    uint32_t *s_dpre = s_fc.excl;   // (free between the traversal of a pass and the next one)
    using AV = acc_t<V>;
    AV *s_vals = reinterpret_cast<AV *>(s_u);                                      // dense: WIN accumulators
    // sparse pass: staged products (column, value) by product number; once every thread holds its
    // products in registers the same memory takes the output (columns, accumulated values) by rank
    // Its memory is laid out per pass: the more windows a stretch spans, the more of the region goes to
    // the bitmap (WIN/8 bytes per window) and its prefix counts (WIN/16), the less to staged products
    // (4 + sizeof(AV) bytes each, in multiples of one product per thread).
    constexpr int OV = WIN / 8 + WIN / 16;
    auto sparse_cap = [](int run) {
        const int c = (HV_REGION - run * OV) / (4 + (int)sizeof(AV)) / HV_THREADS * HV_THREADS;
        return c > HV_HCAP ? HV_HCAP : (c < 0 ? 0 : c);
    };
    int32_t *s_scol = reinterpret_cast<int32_t *>(s_u);
    const int tid = threadIdx.x;
    const size_t stride = (size_t)n_win + 1;

    for (int j = tid; j < WIN; j += HV_THREADS) s_vals[j] = (AV)0;
    for (int j = tid; j < WORDS; j += HV_THREADS) s_dbm[j] = 0u;
    bool dense_clean = true;   // the region is an all-zero dense window
    bool chunk_clean = false;  // the traversal's marks are as wg_flat_chunk_keep leaves them

    for (;;) {
        if (tid == 0) {
            s_row = (long long)atomicAdd(queue, 1ull);
            s_ovf = 0;
        }
        for (int w = tid; w <= n_win; w += HV_THREADS) s_pw[w] = 0u;
        __syncthreads();
        if (s_row >= count) break;   // uniform exit
        const int64_t r = count - 1 - s_row;   // from the end of the list, where the rows with the largest bounds are
        const int64_t row = rows[r];
        const int64_t e0 = a_rp[row], e1 = a_rp[row + 1];
        const int64_t o = out_ptr[row];
        const int64_t cap = out_ptr[row + 1] - o;
        const int64_t ne = e1 - e0;
        long long done = 0;

        // the first HV_THREADS entries of the row stay in registers over all passes
        int32_t ek = 0;
        V ea = V();
        if (tid < ne) { ek = a_col[e0 + tid]; ea = a_val[e0 + tid]; }
        // ---- products of the row per window: one (entry, window) pair per thread and step
        {
            const int de = HV_THREADS / n_win, dw = HV_THREADS % n_win;
            int64_t e = tid / n_win;
            int w = tid % n_win;
            while (e < ne) {
                // four pairs per turn, so that their dependent loads (entry -> boundaries) overlap
                int64_t pe[4];
                int pw[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pe[i] = e; pw[i] = w;
                    e += de;
                    w += dw;
                    if (w >= n_win) { w -= n_win; ++e; }
                }
                int32_t k[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) k[i] = pe[i] < ne ? a_col[e0 + pe[i]] : 0;
                uint32_t d[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t *t = bw + (size_t)k[i] * stride;
                    d[i] = pe[i] < ne ? t[pw[i] + 1] - t[pw[i]] : 0u;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (d[i]) atomicAdd(&s_pw[pw[i] + 1], d[i]);
            }
        }
        __syncthreads();
        {   // counts -> running sums (n_win <= HV_MAXWIN <= HV_THREADS: one window per thread)
            const int mine = tid < n_win ? (int)s_pw[tid + 1] : 0;
            int all;
            const int before = block_exclusive_scan_i32<HV_THREADS>(mine, s_wave, all);
            if (tid < n_win) s_pw[tid + 1] = (uint32_t)(before + mine);
        }
        __syncthreads();

        // ---- walk the windows, pass by pass
        // next pass from window `from` on: a window with more products than a sparse pass can stage (dense),
        // or a run of windows whose products fit the staging memory that is left beside the run's bitmap
        // (sparse); p0 == n_win when nothing is left
        // Every wave plans for itself, 64 windows at a look: lane l holds the running sum behind window
        // from + l, a ballot finds the first window with products, and since the products of a stretch
        // grow with its length while its capacity shrinks, a second ballot finds how far the stretch goes.
        const int lane = tid & (WAVE - 1);
        auto plan = [&](int from, int &p0, int &p1, bool &pdense) {
            p0 = n_win; p1 = n_win; pdense = false;
            for (int x = from; x < n_win; x += WAVE) {   // uniform
                const uint32_t before = s_pw[x];
                const int wl = x + lane;   // this lane's window
                const uint32_t upto = s_pw[(wl < n_win ? wl : n_win - 1) + 1] - before;   // products of [x, wl]
                const unsigned long long some = __ballot(wl < n_win && upto > 0u);
                if (some == 0ull) continue;
                const int k = __ffsll((long long)some) - 1;   // windows x .. x+k-1 are empty
                const unsigned long long fits = __ballot(lane >= k && wl < n_win && upto <= (uint32_t)sparse_cap(lane - k + 1));
                // lanes k, k+1, ... that fit in a row: the stretch
                const unsigned long long stop = ~(fits >> k);
                const int run = stop ? __ffsll((long long)stop) - 1 : WAVE - k;
                p0 = x + k;
                pdense = run == 0;
                p1 = p0 + (run == 0 ? 1 : run);
                return;
            }
        };
        int w, w1;
        bool dense;
        plan(0, w, w1, dense);
        // window boundaries of this thread's entry: those of the next pass are fetched one pass ahead
        const bool have0 = tid < ne;
        const uint32_t *t0 = bw + (size_t)ek * stride;
        uint32_t c_lo = have0 ? t0[w] : 0u, c_hi = have0 ? t0[w1] : 0u;
        while (w < n_win) {
            int nx0, nx1;
            bool nxdense;
            plan(w1, nx0, nx1, nxdense);
            // (no entry has products in the windows skipped between two passes: the next pass starts at c_hi)
            const uint32_t n_hi = have0 ? t0[nx1] : 0u;
            // memory of a sparse pass (see above)
            const int scap = sparse_cap(w1 - w);
            AV *s_sval = reinterpret_cast<AV *>(s_u + (size_t)scap * 4);
            uint16_t *s_hpre = reinterpret_cast<uint16_t *>(s_u + (size_t)scap * (4 + sizeof(AV)));
            uint32_t *s_hbm = reinterpret_cast<uint32_t *>(s_u + (size_t)scap * (4 + sizeof(AV)) + (size_t)(w1 - w) * (WIN / 16));
            const int hwords = (w1 - w) * (WIN / 32);
            // accumulator of this pass
            if (dense) {
                if (!dense_clean) {
                    for (int j = tid; j < WIN; j += HV_THREADS) s_vals[j] = (AV)0;
                    dense_clean = true;
                }
            } else {
                for (int j = tid; j < (w1 - w) * (WIN / 32); j += HV_THREADS) s_hbm[j] = 0u;
                dense_clean = false;
            }
            // (no barrier: the traversal below has barriers of its own before the first product arrives)
            // products of windows [w, w1)
            const int32_t col0 = w * WIN;
            uint32_t staged = 0;   // products of this pass staged so far (sparse pass, uniform)
            auto f = [&](const auto &cj, const auto &cv, uint32_t q0) {
                constexpr int U = sizeof(cj) / sizeof(cj[0]);
                if (dense) {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const unsigned d = (unsigned)(cj[u] - col0);
                        if (cj[u] >= 0 && d < (unsigned)WIN) {   // d is in range for a consistent window table
                            lds_add(&s_vals[d], (AV)cv[u]);
                            // Section 4.1: with many products per output entry most presence bits are set already;
                            // reading the bit first then saves the write (a stale read only costs a redundant OR)
                            const uint32_t bit = 1u << (d & 31);
                            if (!QUERY || !(s_dbm[d >> 5] & bit)) atomicOr(&s_dbm[d >> 5], bit);
                        }
                    }
                } else {
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const uint32_t at = staged + q0 + (uint32_t)u * WAVE + (uint32_t)(tid & (WAVE - 1));
                        const uint32_t d = (uint32_t)(cj[u] - col0);
                        if (cj[u] >= 0 && at < (uint32_t)scap && d < (uint32_t)hwords * 32u) {   // both hold by construction
                            s_scol[at] = cj[u];
                            s_sval[at] = (AV)cv[u];
                            atomicOr(&s_hbm[d >> 5], 1u << (d & 31u));
                        }
                    }
                }
            };
            if (!dense && ne <= HV_THREADS) {
                // ---- sparse pass of a row whose entries fit one chunk: no staging, every product stays in the
                // registers of the thread that fetched it, from the sweep that marks the columns to the sweep
                // that adds the values at their ranks
                constexpr int NBATCH = HV_PPT / FLAT_U;
                static_assert(HV_PPT % FLAT_U == 0, "whole batches");
                int32_t kc[HV_PPT];
                V kv[HV_PPT];
                auto mark = [&](int32_t col) {
                    const uint32_t d = (uint32_t)(col - col0);
                    if (d < (uint32_t)hwords * 32u) atomicOr(&s_hbm[d >> 5], 1u << (d & 31u));   // holds by construction
                };
                bool fits;
                wg_flat_chunk_keep<HV_THREADS, NBATCH>(s_fc, (int)ne, (int64_t)c_lo, c_hi - c_lo, ea, b_col, b_val, kc, kv,
                                                       mark, fits, chunk_clean);
                chunk_clean = true;
                if (!fits && tid == 0) s_ovf = 1;   // cannot happen: passes are planned from the counts
                const int wpt = (hwords + HV_THREADS - 1) / HV_THREADS;   // bitmap words per thread (consecutive)
                int mine = 0;
                for (int q = 0; q < wpt; ++q) {
                    const int j = tid * wpt + q;
                    if (j < hwords) mine += __popc(s_hbm[j]);
                }
                int htotal;
                int run = block_exclusive_scan_i32<HV_THREADS, false>(mine, s_wave, htotal);   // (barrier below)
                for (int q = 0; q < wpt; ++q) {
                    const int j = tid * wpt + q;
                    if (j < hwords) { s_hpre[j] = (uint16_t)run; run += __popc(s_hbm[j]); }
                }
                for (int i = tid; i < htotal; i += HV_THREADS) s_sval[i] = (AV)0;   // (htotal <= products <= scap)
                __syncthreads();
#pragma unroll
                for (int i = 0; i < HV_PPT; ++i) {
                    const uint32_t d = (uint32_t)(kc[i] - col0);
                    if (kc[i] >= 0 && d < (uint32_t)hwords * 32u) {
                        const int rank = (int)s_hpre[d >> 5] + __popc(s_hbm[d >> 5] & ((1u << (d & 31u)) - 1u));
                        s_scol[rank] = kc[i];           // products of one column all write the same id
                        lds_add(&s_sval[rank], (AV)kv[i]);
                    }
                }
                __syncthreads();
                const long long room = cap - done;
                const int n_out = (long long)htotal < room ? htotal : (room > 0 ? (int)room : 0);
                for (int i = tid; i < n_out; i += HV_THREADS) {
                    __builtin_nontemporal_store(s_scol[i], &out_col[o + done + i]);
                    __builtin_nontemporal_store((V)s_sval[i], &out_val[o + done + i]);
                }
                done += htotal;
                __syncthreads();
            } else {
                for (int64_t base = 0; base < ne; base += HV_THREADS) {
                    int32_t k = ek;
                    V a = ea;
                    const bool have = base + tid < ne;
                    if (base > 0 && have) { k = a_col[e0 + base + tid]; a = a_val[e0 + base + tid]; }
                    uint32_t c0 = c_lo, c1 = c_hi;
                    if (base > 0) {
                        c0 = c1 = 0;
                        if (have) {
                            const uint32_t *t = bw + (size_t)k * stride;
                            c0 = t[w];
                            c1 = t[w1];
                        }
                    }
                    const int64_t left = ne - base;
                    staged += wg_flat_chunk<HV_THREADS, true>(s_fc, left < HV_THREADS ? (int)left : HV_THREADS, (int64_t)c0,
                                                              c1 - c0, a, b_col, b_val, f);
                    chunk_clean = false;
                }
                if (dense) {
                    // ---- dense window -> output, in column order
                    const uint32_t word = tid < WORDS ? s_dbm[tid] : 0u;
                    int wtotal;
                    const int ex = block_exclusive_scan_i32<HV_THREADS>(__popc(word), s_wave, wtotal);
                    if (tid < WORDS) s_dpre[tid] = (uint32_t)ex;
                    __syncthreads();
                    // Thread t looks at columns t, t + 1024, ...: in every step the lanes of a wave read
                    // consecutive values (no LDS bank conflicts) and the present ones among them go to
                    // consecutive places of the output (coalesced stores).
                    constexpr int STEPS = WIN / HV_THREADS;   // 16 (fp64) or 32 (fp32)
    #pragma unroll 4
                    for (int i = 0; i < STEPS; ++i) {
                        const int j = i * HV_THREADS + tid;
                        const uint32_t wbits = s_dbm[j >> 5];
                        if ((wbits >> (j & 31)) & 1u) {
                            const long long rank = done + (long long)s_dpre[j >> 5] + __popc(wbits & ((1u << (j & 31)) - 1u));
                            const V val = (V)s_vals[j];
                            s_vals[j] = (AV)0;
                            if (rank < cap) { __builtin_nontemporal_store((int32_t)(col0 + j), &out_col[o + rank]); __builtin_nontemporal_store(val, &out_val[o + rank]); }
                        }
                    }
                    __syncthreads();
                    if (tid < WORDS) s_dbm[tid] = 0u;
                    done += wtotal;
                    __syncthreads();
                } else {
                    // ---- sparse pass: rank of every column = set bits below it in the bitmap of the stretch
                    const int wpt = (hwords + HV_THREADS - 1) / HV_THREADS;   // bitmap words per thread (consecutive)
                    int mine = 0;
                    for (int q = 0; q < wpt; ++q) {
                        const int j = tid * wpt + q;
                        if (j < hwords) mine += __popc(s_hbm[j]);
                    }
                    int htotal;
                    int run = block_exclusive_scan_i32<HV_THREADS, false>(mine, s_wave, htotal);   // (barrier below)
                    for (int q = 0; q < wpt; ++q) {
                        const int j = tid * wpt + q;
                        if (j < hwords) { s_hpre[j] = (uint16_t)run; run += __popc(s_hbm[j]); }
                    }
                    __syncthreads();
                    // every thread takes its share of the staged products into registers, with their ranks
                    if (staged > (uint32_t)scap) staged = scap;   // cannot happen: passes are planned from the counts
                    int32_t pc[HV_PPT];
                    AV pv[HV_PPT];
                    int pr[HV_PPT];
    #pragma unroll
                    for (int i = 0; i < HV_PPT; ++i) {
                        const uint32_t at = (uint32_t)i * HV_THREADS + tid;
                        pc[i] = -1; pv[i] = AV(); pr[i] = 0;
                        if (at < staged) {
                            pc[i] = s_scol[at];
                            pv[i] = s_sval[at];
                            s_sval[at] = (AV)0;   // (htotal <= staged: the values of the output start from zero)
                            const uint32_t d = (uint32_t)(pc[i] - col0);
                            pr[i] = (int)s_hpre[d >> 5] + __popc(s_hbm[d >> 5] & ((1u << (d & 31u)) - 1u));
                        }
                    }
                    __syncthreads();
                    // the staging memory becomes the output of the pass: columns and values by rank
    #pragma unroll
                    for (int i = 0; i < HV_PPT; ++i) {
                        if (pc[i] >= 0) {
                            s_scol[pr[i]] = pc[i];          // products of one column all write the same id
                            lds_add(&s_sval[pr[i]], pv[i]);
                        }
                    }
                    __syncthreads();
                    const long long room = cap - done;
                    const int n_out = (long long)htotal < room ? htotal : (room > 0 ? (int)room : 0);
                    for (int i = tid; i < n_out; i += HV_THREADS) {
                        __builtin_nontemporal_store(s_scol[i], &out_col[o + done + i]);
                        __builtin_nontemporal_store((V)s_sval[i], &out_val[o + done + i]);
                    }
                    done += htotal;
                    __syncthreads();
                }
            }
            c_lo = c_hi; c_hi = n_hi;
            w = nx0; w1 = nx1; dense = nxdense;
        }
        if (tid == 0) row_nnz[row] = (s_ovf || done > cap) ? -1 : (int32_t)done;
        __syncthreads();
    }
}

// Positions of the column-window boundaries inside every row of B:
// bw[k*(n_win+1)+w] = first position p in row k with col[p] >= w*win (row end if none).
// One 16-lane group per row; a row of WT_LONG or more entries is left to the whole workgroup (every entry is
// looked at on its own, together with its predecessor), which takes the long rows of its 16 one after the other:
// the longest row of a power-law matrix, walked by 16 lanes, was most of the kernel's time.
// flags |= 8 when a row is not sorted ascending.
constexpr int WT_LONG = 1024;
__global__ void __launch_bounds__(256)
k_window_table(const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, int64_t rows, int win_log2,
               int n_win, int64_t long_from, uint32_t *__restrict__ bw, int32_t *flags)
{
    __shared__ long long s_long[16];
    __shared__ int s_nlong;
    const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t k = gt >> 4;
    const int sub = (int)(gt & 15);
    if (threadIdx.x == 0) s_nlong = 0;
    __syncthreads();
    bool unsorted = false;
    // entries first, first + step, ... of row r (positions p0 .. p1 - 1, p0 < p1), four per lane and turn
    // (unconditional reads, index clamped), so that a long row is not bound by the latency of one load after the other
    auto walk = [&](int64_t r, int64_t p0, int64_t p1, int first, int step) {
        uint32_t *t = bw + (size_t)r * ((size_t)n_win + 1);
        for (int64_t q = p0 + first; q < p1; q += 4 * (int64_t)step) {
            int32_t c[4], cp[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t p = q + (int64_t)step * i;
                const int64_t pc = p < p1 ? p : p1 - 1;
                c[i] = b_col[pc];
                cp[i] = b_col[pc > p0 ? pc - 1 : p0];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t p = q + (int64_t)step * i;
                if (p >= p1) break;
                const int wc = c[i] >> win_log2;
                int wprev = -1;
                if (p > p0) {
                    unsorted |= cp[i] > c[i];
                    wprev = cp[i] >> win_log2;
                }
                for (int w = wprev + 1; w <= wc; ++w) t[w] = (uint32_t)p;
                if (p == p1 - 1)
                    for (int w = wc + 1; w <= n_win; ++w) t[w] = (uint32_t)p1;
            }
        }
    };
    if (k < rows) {
        const int64_t p0 = b_rp[k], p1 = b_rp[k + 1];
        if (p0 == p1) {
            uint32_t *t = bw + (size_t)k * ((size_t)n_win + 1);
            for (int w = sub; w <= n_win; w += 16) t[w] = (uint32_t)p0;
        } else if (p1 - p0 >= long_from) {
            if (sub == 0) s_long[atomicAdd(&s_nlong, 1)] = k;
        } else {
            walk(k, p0, p1, sub, 16);
        }
    }
    __syncthreads();
    const int nlong = s_nlong;
    for (int i = 0; i < nlong; ++i) {   // uniform
        const int64_t r = s_long[i];
        walk(r, b_rp[r], b_rp[r + 1], (int)threadIdx.x, 256);
    }
    if (unsorted) atomicOr(flags, 8);
}

hipError_t launch_window_table(const Csr &B, int dtype, uint32_t *bw, int *n_win_out, int32_t *flags, hipStream_t s)
{
    (void)dtype;
    const int win_log2 = ilog2_const(HV_REGION / 8);   // (both value types accumulate in 8 bytes)
    const int n_win = (int)((B.cols + (1ll << win_log2) - 1) >> win_log2);
    *n_win_out = n_win;
    if (B.rows == 0) return hipSuccess;
    const int64_t threads = B.rows * 16;
    // ("long" is relative: 1024 entries or eight times the average row, whichever is more)
    const double avg = (double)B.nnz / (double)B.rows;
    const int64_t long_from = 8.0 * avg > (double)WT_LONG ? (int64_t)(8.0 * avg) : (int64_t)WT_LONG;
    hipLaunchKernelGGL(k_window_table, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, B.rp, B.col, B.rows,
                       win_log2, n_win, long_from, bw, flags);
    return hipGetLastError();
}

int heavy_workgroups_per_cu() { return HV_WG_PER_CU; }

int dense_window_count(int64_t n_cols, int dtype)
{
    (void)dtype;
    const int win_log2 = ilog2_const(HV_REGION / 8);   // (both value types accumulate in 8 bytes)
    return (int)((n_cols + (1ll << win_log2) - 1) >> win_log2);
}

// ======================================================= global kernel ====
// The table of a row lives in this workgroup's region of global memory
// (tables are EMPTY / zero between rows).  Rows are emitted in order through
// an LDS bitmap over windows of 512 K columns, which also restores the table.
constexpr int GL_THREADS = 1024;
constexpr int GL_WIN = 524288;
constexpr int GL_WORDS = GL_WIN / 32;   // 16384

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
    __shared__ WgChunk<V, GL_THREADS> s_fc;
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
        if (tid == 0) { s_ovf = 0; s_min = 0x7fffffff; s_max = -1; }
        __syncthreads();

        int kmin = 0x7fffffff, kmax = -1;
        wg_traverse<GL_THREADS, true>(a_col, a_val, a_rp[row], a_rp[row + 1],
                                      [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                      b_col, b_val, s_fc, [&](const auto &cj, const auto &cv) {
                                          constexpr int U = sizeof(cj) / sizeof(cj[0]);
                                          const uint32_t mask = (1u << bits) - 1u;
                                          uint32_t h[U], st[U];
                                          bool pend[U];
                                          bool any = false;
#pragma unroll
                                          for (int u = 0; u < U; ++u) {
                                              pend[u] = cj[u] >= 0;
                                              h[u] = table_hash(cj[u], bits);
                                              st[u] = table_step(cj[u], bits);
                                              any |= pend[u];
                                              if (pend[u]) {
                                                  kmin = cj[u] < kmin ? cj[u] : kmin;
                                                  kmax = cj[u] > kmax ? cj[u] : kmax;
                                              }
                                          }
                                          uint32_t rounds = 0;
                                          while (any) {   // all unresolved products probe together: their L2 round trips overlap
                                              int32_t old[U];
#pragma unroll
                                              for (int u = 0; u < U; ++u)
                                                  if (pend[u]) old[u] = atomicCAS(&gk[h[u]], EMPTY_KEY, cj[u]);
                                              any = false;
#pragma unroll
                                              for (int u = 0; u < U; ++u) {
                                                  if (pend[u]) {
                                                      if (old[u] == EMPTY_KEY || old[u] == cj[u]) {
                                                          pend[u] = false;
                                                          l2_add(&gv[h[u]], cv[u]);
                                                      } else {
                                                          h[u] = (h[u] + st[u]) & mask;
                                                          any = true;
                                                      }
                                                  }
                                              }
                                              if (any && ++rounds > mask) { s_ovf = 1; break; }
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
static hipError_t dispatch(const Csr &A, const Csr &B, const NumLaunch &l, int /*gb_log2*/, hipStream_t s)
{
    if (l.count <= 0) return hipSuccess;
    const V *av = static_cast<const V *>(A.val);
    const V *bv = static_cast<const V *>(B.val);
    V *ov = static_cast<V *>(l.out_val);
#define OCEAN_WG_BF(BITS, THREADS, BF)                                                                              \
    hipLaunchKernelGGL((k_numeric_wg<V, BITS, THREADS, BF>), dim3((unsigned)l.count), dim3(THREADS), 0, s, A.rp, A.col, \
                       av, B.rp, B.col, bv, l.rows, l.count, l.out_ptr, l.out_col, ov, l.row_nnz)
#define OCEAN_WG(BITS, THREADS) OCEAN_WG_BF(BITS, THREADS, 1)
    switch (l.bin) {
    case NB_E16:
    case NB_G8: {
        const int64_t blocks = (l.count + 31) / 32;
        hipLaunchKernelGGL((k_numeric_group<V, 8, 5>), dim3((unsigned)blocks), dim3(256), 0, s, A.rp, A.col, av, B.rp, B.col,
                           bv, l.rows, l.count, l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    }
    case NB_G16: {
        const int64_t blocks = (l.count + 15) / 16;
        hipLaunchKernelGGL((k_numeric_group<V, 16, 6>), dim3((unsigned)blocks), dim3(256), 0, s, A.rp, A.col, av, B.rp, B.col,
                           bv, l.rows, l.count, l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    }
#define OCEAN_WAVE(BITS, R)                                                                                        \
    hipLaunchKernelGGL((k_numeric_wave<V, BITS, R>), dim3((unsigned)((l.count + (R) - 1) / (R))), dim3(WAVE * (R)), 0, s, A.rp, \
                       A.col, av, B.rp, B.col, bv, l.rows, l.count, l.out_ptr, l.out_col, ov, l.row_nnz)
    case NB_W64: OCEAN_WAVE(8, 4); break;
    // a wave per row while the rows of the bin are light; a workgroup per row when they hold many products each
    // (a wave per row was measured for the 512- and 1024-slot bins too: 1.3 - 1.6 x slower than a workgroup per row)
    case NB_S512:
        if (l.fine_buckets) OCEAN_WG_BF(9, 128, 4);
        else OCEAN_WG(9, 128);
        break;
    case NB_S1K:
        if (l.fine_buckets) OCEAN_WG_BF(10, 256, 2);
        else OCEAN_WG(10, 256);
        break;
    case NB_S2K: OCEAN_WG(11, 512); break;
    case NB_S4K: OCEAN_WG(12, 512); break;
    case NB_S8K: OCEAN_WG(13, 1024); break;
    case NB_DSPAN:
        if (l.cmin == nullptr) return hipErrorInvalidValue;
        if (l.query_bitmap)
            hipLaunchKernelGGL((k_numeric_dspan<V, true>), dim3((unsigned)l.count), dim3(DS_THREADS), 0, s, A.rp, A.col, av, B.rp,
                               B.col, bv, l.rows, l.count, l.cmin, l.out_ptr, l.out_col, ov, l.row_nnz);
        else
            hipLaunchKernelGGL((k_numeric_dspan<V, false>), dim3((unsigned)l.count), dim3(DS_THREADS), 0, s, A.rp, A.col, av, B.rp,
                               B.col, bv, l.rows, l.count, l.cmin, l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    case NB_HYBRID:
        if (l.bw != nullptr) return hipErrorInvalidValue;   // such rows go with the last bin
        else
            hipLaunchKernelGGL((k_numeric_hybrid<V>), dim3((unsigned)l.n_wg), dim3(HY_THREADS), 0, s, A.rp, A.col, av,
                               B.rp, B.col, bv, l.rows, l.count, l.queue, static_cast<V *>(l.slab),
                               static_cast<uint2 *>(l.pairs), l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    case NB_GLOBAL:
        if (l.bw != nullptr && l.query_bitmap)
            hipLaunchKernelGGL((k_numeric_heavy<V, true>), dim3((unsigned)l.n_wg), dim3(HV_THREADS), 0, s, A.rp, A.col, av, l.bw,
                               l.n_win, B.col, bv, l.rows, l.count, l.queue, l.out_ptr, l.out_col, ov, l.row_nnz);
        else if (l.bw != nullptr)
            hipLaunchKernelGGL((k_numeric_heavy<V, false>), dim3((unsigned)l.n_wg), dim3(HV_THREADS), 0, s, A.rp, A.col, av, l.bw,
                               l.n_win, B.col, bv, l.rows, l.count, l.queue, l.out_ptr, l.out_col, ov, l.row_nnz);
        else
            hipLaunchKernelGGL((k_numeric_global<V>), dim3((unsigned)l.n_wg), dim3(GL_THREADS), 0, s, A.rp, A.col, av,
                               B.rp, B.col, bv, l.rows, l.count, l.queue, l.gkeys, static_cast<V *>(l.gvals), l.gbits,
                               l.coef, l.out_ptr, l.out_col, ov, l.row_nnz);
        break;
    default: return hipErrorInvalidValue;
    }
#undef OCEAN_WG
#undef OCEAN_WG_BF
#undef OCEAN_WAVE
    return hipGetLastError();
}

hipError_t launch_numeric_bin(const Csr &A, const Csr &B, int dtype, const NumLaunch &l, int gb_log2, hipStream_t s)
{
    return dtype == OCEAN_F64 ? dispatch<double>(A, B, l, gb_log2, s) : dispatch<float>(A, B, l, gb_log2, s);
}

}  // namespace ocean
