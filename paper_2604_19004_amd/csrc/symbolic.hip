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

using NoVal = unsigned char;   // the symbolic pass carries no values

// Insert a batch of column ids into a key-only LDS table and return how many
// were new.  Double hashing, and every lane walks its own ids at its own pace
// (one compare-and-swap per lane and round), so the wave-wide loop runs for the
// largest per-lane sum of probes.  Valid ids come first in a batch.
// A table sized from the product count cannot fill up.  A table sized from a
// guess (assisted binning, Section 4.1) can: then CAPPED gives up on an id after
// PROBE_CAP probes - at the load such a table is meant for (0.8) a longer probe
// sequence is a one-in-a-million event, in a table about to fill up it is the
// rule and would cost thousands of probes per id - and sets ovf; the caller
// redoes such a row with a table sized from its product count.
constexpr uint32_t PROBE_CAP = 64;
template <int BITS, bool CAPPED, int U>
__device__ __forceinline__ int lds_count_new_batch(int32_t *keys, const int32_t (&cj)[U], bool &ovf)
{
    constexpr uint32_t MASK = (1u << BITS) - 1u;
    constexpr uint32_t LIMIT = CAPPED && PROBE_CAP < MASK ? PROBE_CAP : MASK;
    int idx = 0, fresh = 0;
    int32_t key = cj[0];
    uint32_t h = table_hash(key, BITS);
    uint32_t step = table_step(key, BITS);
    uint32_t rounds = 0;
    while (key >= 0) {
        const int32_t old = atomicCAS(&keys[h], EMPTY_KEY, key);
        if (old == EMPTY_KEY || old == key) {
            fresh += (old == EMPTY_KEY);
            ++idx;
            key = -1;
#pragma unroll
            for (int u = 1; u < U; ++u)
                if (idx == u) key = cj[u];
            h = table_hash(key, BITS);
            step = table_step(key, BITS);
            rounds = 0;
        } else {
            h = (h + step) & MASK;
            if (++rounds > LIMIT) {   // (a table sized from the product count cannot fill up)
                if (CAPPED) ovf = true;
                key = -1;
            }
        }
    }
    return fresh;
}

// ---------------------------------------------------------- group kernel
template <bool CAPPED>
__global__ void __launch_bounds__(256)
k_symbolic_group(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
                 const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col,
                 const int32_t *__restrict__ rows, int64_t count, int32_t *__restrict__ nnz_out)
{
    constexpr int G = 16;
    constexpr int BITS = 6;
    constexpr int SLOTS = 1 << BITS;
    constexpr int R = 256 / G;
    __shared__ int32_t s_keys[R * SLOTS];
    __shared__ FlatChunk<NoVal, G> s_fc[R];
    const int rl = threadIdx.x / G;
    const int sub = threadIdx.x % G;
    int32_t *keys = s_keys + rl * SLOTS;
    const int64_t r = (int64_t)blockIdx.x * R + rl;
    const bool live = r < count;
    const int64_t row = live ? rows[r] : 0;
    for (int s = sub; s < SLOTS; s += G) keys[s] = EMPTY_KEY;
    wave_sync();
    int fresh = 0;
    bool ovf = false;
    const int64_t e0 = live ? a_rp[row] : 0;
    const int64_t e1 = live ? a_rp[row + 1] : 0;
    auto f = [&](const auto &cj, const auto &) { if (!CAPPED || !ovf) fresh += lds_count_new_batch<BITS, CAPPED>(keys, cj, ovf); };
    const int chunks = (int)wave_max_u32((uint32_t)((e1 - e0 + G - 1) / G));   // (uniform: the rows of a wave advance together)
    for (int ch = 0; ch < chunks; ++ch) {
        const int64_t e = e0 + (int64_t)ch * G + sub;
        int64_t p0 = 0;
        uint32_t len = 0;
        if (e < e1) {
            const int64_t k = a_col[e];
            p0 = b_rp[k];
            len = (uint32_t)(b_rp[k + 1] - p0);
        }
        group_flat<G, false>(s_fc[rl], p0, len, NoVal(), b_col, (const NoVal *)nullptr, f);
    }
    fresh = (int)group_sum_u32<G>((uint32_t)fresh);
    const bool ovf_any = CAPPED && group_sum_u32<G>((uint32_t)ovf) != 0u;
    if (live && sub == 0) nnz_out[row] = ovf_any ? -1 : fresh;
}

// ----------------------------------------------------------- wave kernel
template <bool CAPPED>
__global__ void __launch_bounds__(256)
k_symbolic_wave(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
                const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col,
                const int32_t *__restrict__ rows, int64_t count, int32_t *__restrict__ nnz_out)
{
    constexpr int BITS = 8;
    constexpr int SLOTS = 1 << BITS;
    __shared__ int32_t s_keys[4 * SLOTS];
    __shared__ FlatChunk<NoVal, WAVE> s_fc[4];
    const int rl = threadIdx.x / WAVE;
    const int sub = lane_id();
    int32_t *keys = s_keys + rl * SLOTS;
    const int64_t r = (int64_t)blockIdx.x * 4 + rl;
    if (r >= count) return;   // no workgroup barrier below
    const int64_t row = rows[r];
    for (int s = sub; s < SLOTS; s += WAVE) keys[s] = EMPTY_KEY;
    wave_sync();
    int fresh = 0;
    bool ovf = false;
    wave_traverse<false>(a_col, (const NoVal *)nullptr, a_rp[row], a_rp[row + 1],
                         [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                         b_col, (const NoVal *)nullptr, s_fc[rl],
                         [&](const auto &cj, const auto &) { if (!CAPPED || !ovf) fresh += lds_count_new_batch<BITS, CAPPED>(keys, cj, ovf); });
    fresh = (int)wave_sum_u32((uint32_t)fresh);
    const bool ovf_any = CAPPED && __ballot(ovf) != 0ull;
    if (sub == 0) nnz_out[row] = ovf_any ? -1 : fresh;
}

// ------------------------------------------------------ workgroup kernel
template <int BITS, int THREADS, bool CAPPED>
__global__ void __launch_bounds__(THREADS)
k_symbolic_wg(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
              const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col,
              const int32_t *__restrict__ rows, int64_t count, int32_t *__restrict__ nnz_out)
{
    constexpr int SLOTS = 1 << BITS;
    __shared__ int32_t s_keys[SLOTS];
    __shared__ WgChunk<NoVal, THREADS> s_fc;
    __shared__ int s_count, s_ovf;
    const int tid = threadIdx.x;
    const int64_t r = blockIdx.x;
    if (r >= count) return;
    const int64_t row = rows[r];
    for (int s = tid; s < SLOTS; s += THREADS) s_keys[s] = EMPTY_KEY;
    if (tid == 0) { s_count = 0; s_ovf = 0; }
    __syncthreads();
    int fresh = 0;
    bool ovf = false;
    wg_traverse<THREADS, false>(a_col, (const NoVal *)nullptr, a_rp[row], a_rp[row + 1],
                                [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                b_col, (const NoVal *)nullptr, s_fc,
                                [&](const auto &cj, const auto &) { if (!CAPPED || !ovf) fresh += lds_count_new_batch<BITS, CAPPED>(s_keys, cj, ovf); });
    fresh = (int)wave_sum_u32((uint32_t)fresh);
    if (lane_id() == 0 && fresh) atomicAdd(&s_count, fresh);
    if (CAPPED && ovf) s_ovf = 1;
    __syncthreads();
    if (tid == 0) nnz_out[row] = (CAPPED && s_ovf) ? -1 : s_count;
}

// --------------------------------------------------------- bitmap kernel
constexpr int BM_THREADS = 1024;
constexpr int BM_U = 16;                 // column ids per lane and batch (R-MAT: 16.2 ms against 16.9 with 8, 20.9 with 4)
constexpr int BM_WIN = 1 << 20;          // columns per window
constexpr int BM_WORDS = BM_WIN / 32;    // 32768 words = 128 KB

// ONE_WINDOW: B has at most BM_WIN columns, so every column id falls into the one window.
// QUERY: a column's bit is read first and set only when it is clear (Section 4.1).
template <bool ONE_WINDOW, bool QUERY>
__global__ void __launch_bounds__(BM_THREADS)
k_symbolic_bitmap(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col,
                  const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col,
                  const int32_t *__restrict__ rows, int64_t count, int64_t n_cols,
                  unsigned long long *queue, int32_t *__restrict__ nnz_out)
{
    __shared__ __align__(16) uint32_t s_bm[BM_WORDS];
    __shared__ WgChunk<NoVal, BM_THREADS> s_fc;
    // Rows come from a shared counter.  The chain counter -> row id -> offsets of the row -> entries -> their
    // segments of B is five memory round trips before the first column id of a row can be asked for, so it runs
    // ahead of the work, one link per turn: at the start of a turn the ticket of the row six turns ahead is
    // drawn and the row id (four ahead), the offsets (three), the first BM_THREADS entries (two) and their
    // segments (one) are asked for, all of which arrive under the traversal of the current row.  s_ticket: ring
    // of eight tickets (count >= 1); a ticket is first read two turns after it was stored, behind the barriers
    // of the turn between, and the row counts alternate between two cells, so a turn ends without a barrier.
    __shared__ unsigned long long s_ticket[8];
    __shared__ int s_count[2];
    const int tid = threadIdx.x;
    for (int s = tid; s < BM_WORDS; s += BM_THREADS) s_bm[s] = 0u;
    if (tid == 0) {
        for (int j = 0; j < 6; ++j) s_ticket[j] = atomicAdd(queue, 1ull);
        s_count[0] = s_count[1] = 0;
    }
    __syncthreads();
    // a ticket beyond the list stands for no row; its loads use the list's first row instead
    auto row_of = [&](unsigned turn) {
        const unsigned long long t = s_ticket[turn & 7u];
        return (int64_t)rows[t < (unsigned long long)count ? count - 1 - (int64_t)t : (int64_t)0];   // (the largest bounds are at the end)
    };
    auto entry_of = [&](int64_t f0, int64_t f1) { return f0 + tid < f1 ? a_col[f0 + tid] : (int32_t)-1; };
    auto segment_of = [&](int32_t k, int64_t &p0, uint32_t &len) {
        p0 = 0; len = 0u;
        if (k >= 0) {
            p0 = b_rp[k];
            len = (uint32_t)(b_rp[k + 1] - p0);
        }
    };
    int64_t row = row_of(0), row1 = row_of(1), row2 = row_of(2), row3 = row_of(3);
    int64_t e0 = a_rp[row], e1 = a_rp[row + 1];
    int64_t e0_1 = a_rp[row1], e1_1 = a_rp[row1 + 1];
    int64_t e0_2 = a_rp[row2], e1_2 = a_rp[row2 + 1];
    int32_t k1 = entry_of(e0_1, e1_1);
    int64_t fp0;
    uint32_t flen;
    segment_of(entry_of(e0, e1), fp0, flen);
    auto mark = [&](const auto &cj, uint32_t w0, auto all_valid) {
        constexpr int U = sizeof(cj) / sizeof(cj[0]);
        constexpr bool ALL = decltype(all_valid)::value;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // (32-bit arithmetic: a column before the window wraps to a large number)
            const uint32_t d = ONE_WINDOW ? (uint32_t)cj[u] : (uint32_t)cj[u] - w0;
            // Only the number of set bits matters, so neighbouring columns (the sorted entries of one row of
            // B in neighbouring lanes) go to neighbouring words, i.e. different LDS banks, not to one word.
            if ((ALL || cj[u] >= 0) && (ONE_WINDOW || d < (uint32_t)BM_WIN)) {
                const uint32_t bit = 1u << (d / (uint32_t)BM_WORDS);
                uint32_t *word = &s_bm[d & (uint32_t)(BM_WORDS - 1)];
                if (!QUERY || !(*word & bit)) atomicOr(word, bit);
            }
        }
    };
    for (unsigned turn = 0;; ++turn) {
        if (s_ticket[turn & 7u] >= (unsigned long long)count) break;   // uniform exit (tickets only grow)
        unsigned long long drawn = 0;
        if (tid == 0) drawn = atomicAdd(queue, 1ull);                  // ticket of turn + 6
        const int64_t row4 = row_of(turn + 4u);
        const int64_t e0_3 = a_rp[row3], e1_3 = a_rp[row3 + 1];
        const int32_t k2 = entry_of(e0_2, e1_2);
        int64_t fp0_1;
        uint32_t flen_1;
        segment_of(k1, fp0_1, flen_1);
        const int64_t ne = e1 - e0;
        for (int64_t w0 = 0; w0 < n_cols; w0 += BM_WIN) {
            auto f = [&](const auto &cj, const auto &, auto... tag) {
                mark(cj, (uint32_t)w0, std::bool_constant<(std::is_same_v<decltype(tag), AllValid> || ...)>{});
            };
            if (ne > 0)
                wg_flat_chunk<BM_THREADS, false, BM_U>(s_fc, ne < BM_THREADS ? (int)ne : BM_THREADS, fp0, flen, NoVal(), b_col,
                                                       (const NoVal *)nullptr, f);
            if (ne > BM_THREADS)
                wg_traverse<BM_THREADS, false, BM_U>(a_col, (const NoVal *)nullptr, e0 + BM_THREADS, e1,
                                                     [&](int32_t k, int64_t &p0, int64_t &len) { p0 = b_rp[k]; len = b_rp[k + 1] - p0; },
                                                     b_col, (const NoVal *)nullptr, s_fc, f);
            // (both end with a barrier)  count and clear the window, 16 bytes per thread and step
            int c = 0;
            uint4 *bm4 = reinterpret_cast<uint4 *>(s_bm);
#pragma unroll
            for (int s = 0; s < BM_WORDS / 4 / BM_THREADS; ++s) {
                const uint4 x = bm4[s * BM_THREADS + tid];
                c += __popc(x.x) + __popc(x.y) + __popc(x.z) + __popc(x.w);
                bm4[s * BM_THREADS + tid] = make_uint4(0u, 0u, 0u, 0u);
            }
            c = (int)wave_sum_u32((uint32_t)c);
            if (lane_id() == 0 && c) atomicAdd(&s_count[turn & 1u], c);
            __syncthreads();
        }
        if (tid == 0) {
            nnz_out[row] = s_count[turn & 1u];
            s_count[turn & 1u] = 0;               // (next used two turns from now)
            s_ticket[(turn + 6u) & 7u] = drawn;   // (its slot held the ticket of two turns ago)
        }
        row = row1; row1 = row2; row2 = row3; row3 = row4;
        e0 = e0_1; e1 = e1_1;
        e0_1 = e0_2; e1_1 = e1_2;
        e0_2 = e0_3; e1_2 = e1_3;
        k1 = k2;
        fp0 = fp0_1; flen = flen_1;
    }
}

// -------------------------------------------------------------- dispatch
hipError_t launch_symbolic_bin(const Csr &A, const Csr &B, const SymLaunch &l, int /*gb_log2*/, int32_t *nnz_out,
                               int n_wg, unsigned long long *queue, hipStream_t s)
{
    if (l.count <= 0) return hipSuccess;
#define OCEAN_SYM_WG(BITS, THREADS)                                                                               \
    do {                                                                                                          \
        if (l.may_overflow)                                                                                       \
            hipLaunchKernelGGL((k_symbolic_wg<BITS, THREADS, true>), dim3((unsigned)l.count), dim3(THREADS), 0, s,  \
                               A.rp, A.col, B.rp, B.col, l.rows, l.count, nnz_out);                               \
        else                                                                                                      \
            hipLaunchKernelGGL((k_symbolic_wg<BITS, THREADS, false>), dim3((unsigned)l.count), dim3(THREADS), 0, s, \
                               A.rp, A.col, B.rp, B.col, l.rows, l.count, nnz_out);                               \
    } while (0)
    switch (l.bin) {
    case SB_G16:
        if (l.may_overflow)
            hipLaunchKernelGGL(k_symbolic_group<true>, dim3((unsigned)((l.count + 15) / 16)), dim3(256), 0, s, A.rp, A.col,
                               B.rp, B.col, l.rows, l.count, nnz_out);
        else
            hipLaunchKernelGGL(k_symbolic_group<false>, dim3((unsigned)((l.count + 15) / 16)), dim3(256), 0, s, A.rp, A.col,
                               B.rp, B.col, l.rows, l.count, nnz_out);
        break;
    case SB_W64:
        if (l.may_overflow)
            hipLaunchKernelGGL(k_symbolic_wave<true>, dim3((unsigned)((l.count + 3) / 4)), dim3(256), 0, s, A.rp, A.col, B.rp,
                               B.col, l.rows, l.count, nnz_out);
        else
            hipLaunchKernelGGL(k_symbolic_wave<false>, dim3((unsigned)((l.count + 3) / 4)), dim3(256), 0, s, A.rp, A.col, B.rp,
                               B.col, l.rows, l.count, nnz_out);
        break;
    case SB_S1K: OCEAN_SYM_WG(10, 64); break;    // (rect: 64 threads 0.68 ms, 128 0.76, 256 1.08 for the whole stage)
    case SB_S4K: OCEAN_SYM_WG(12, 256); break;   // (clustered: 256 threads 1.16 ms, 128 1.23, 512 1.40)
    case SB_S16K: OCEAN_SYM_WG(14, 1024); break;
    case SB_S32K: OCEAN_SYM_WG(15, 1024); break;
    case SB_BITMAP: {
#define OCEAN_SYM_BM(ONE, QUERY)                                                                                  \
    hipLaunchKernelGGL((k_symbolic_bitmap<ONE, QUERY>), dim3((unsigned)n_wg), dim3(BM_THREADS), 0, s, A.rp, A.col, B.rp,  \
                       B.col, l.rows, l.count, B.cols, queue, nnz_out)
        const bool one = B.cols <= BM_WIN;
        if (one && l.query_bitmap) OCEAN_SYM_BM(true, true);
        else if (one) OCEAN_SYM_BM(true, false);
        else if (l.query_bitmap) OCEAN_SYM_BM(false, true);
        else OCEAN_SYM_BM(false, false);
#undef OCEAN_SYM_BM
        break;
    }
    default: return hipErrorInvalidValue;
    }
#undef OCEAN_SYM_WG
    return hipGetLastError();
}

}  // namespace ocean
