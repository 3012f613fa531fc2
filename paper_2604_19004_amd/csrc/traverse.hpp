// Traversal of the intermediate products of one row of C = A*B (Gustavson's two
// nested loops, paper Section 2.1) by a whole workgroup, one wave or a group
// of lanes.
//
// What matters is that all 64 lanes of a wave carry a product in every
// instruction and that independent memory operations are in flight together.
// Rows of B referenced by one row of A differ wildly in length on power-law
// matrices; a fixed "lanes per row of B" mapping leaves most lanes idle.
// Therefore:
//   * a workgroup FLATTENS the products of a row: it takes up to THREADS
//     entries A_ik, prefix-sums the lengths of their rows of B, and every wave
//     handles one contiguous span of the concatenated segments, 64 consecutive
//     products per load instruction (consecutive lanes mostly fall into one row
//     of B, so the loads stay coalesced); the entry of a product is found by a
//     bitmap rank or a binary search over the prefix sums kept in LDS;
//   * a wave or a group of 8 or 16 lanes that owns a short row does the same
//     over its 64, 8 or 16 entries; rows of B of T_LONG or more entries are
//     walked 64-wide there.
// Prefix sums inside a wave use DPP moves, not LDS permutes.
// Products reach the accumulator in batches: f(cj, cv) receives U column ids
// (negative = none) and values a*b per lane, so that the accumulator's own
// dependent LDS round trips (hash probes) overlap across the batch.
#pragma once

#include <type_traits>

#include "ocean_internal.hpp"

namespace ocean {

constexpr int T_LONG = 128;
constexpr int FLAT_U = 4;

// Third argument of an accumulator's batch function when every column id of the batch is a real one.
struct AllValid {};
// 16 bytes of column ids at any 4-byte boundary (one load instruction).
struct alignas(4) Int4U { int32_t v[4]; };

// Products p0 + lane, p0 + lane + STRIDE, ... of one segment, UNROLL loads in flight per lane.
template <int STRIDE, int UNROLL, bool HAS_VAL, typename V, typename F>
__device__ __forceinline__ void exec_segment(const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
                                             int64_t p0, int64_t len, int lane, V a, F &f)
{
    const int64_t end = p0 + len;
    for (int64_t base = p0 + lane; base < end; base += (int64_t)STRIDE * UNROLL) {
        int32_t cj[UNROLL];
        V cv[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int64_t p = base + (int64_t)u * STRIDE;
            const bool ok = p < end;
            cj[u] = ok ? b_col[p] : -1;
            if constexpr (HAS_VAL) cv[u] = ok ? a * b_val[p] : V();
            else cv[u] = V();
        }
        f(cj, cv);
    }
}

// LDS scratch of one flattened chunk: per entry the exclusive prefix of the
// lengths, the position of its first product minus that prefix, and A's value.
template <typename V, int G>
struct FlatChunk {
    uint32_t excl[G];
    long long pbase[G];
    V a[G];
};

// G lanes (8, 16 or the 64 of a wave; consecutive lanes of one wave) flatten the G segments
// (p0, len, a) they hold, len < 2^24.  Every lane of the group calls it.
template <int G, bool HAS_VAL, typename V, typename F>
__device__ __forceinline__ void group_flat(FlatChunk<V, G> &c, int64_t p0, uint32_t len, V a,
                                           const int32_t *__restrict__ b_col, const V *__restrict__ b_val, F &f)
{
    const int sub = lane_id() & (G - 1);
    uint32_t incl, total;
    if constexpr (G == WAVE) {
        incl = wave_inclusive_scan_u32(len);
        total = wave_read_lane_u32(incl, WAVE - 1);
    } else {
        incl = group_inclusive_scan_u32<G>(len, sub);
        total = group_sum_u32<G>(len);
    }
    if (G == WAVE && total == 0) return;   // uniform for a whole wave
    c.excl[sub] = incl - len;
    c.pbase[sub] = (long long)p0 - (long long)(incl - len);
    c.a[sub] = a;
    wave_sync();
    for (uint32_t q0 = 0; q0 < total; q0 += G * FLAT_U) {
        int32_t cj[FLAT_U];
        V cv[FLAT_U];
#pragma unroll
        for (int u = 0; u < FLAT_U; ++u) {
            const uint32_t q = q0 + u * G + sub;
            const bool ok = q < total;
            int pos = 0;
#pragma unroll
            for (int step = G >> 1; step > 0; step >>= 1)
                if (c.excl[pos + step] <= q) pos += step;   // last entry starting at or before q (skips empty ones)
            const int64_t p = c.pbase[pos] + (long long)q;
            cj[u] = ok ? b_col[p] : -1;
            if constexpr (HAS_VAL) cv[u] = ok ? c.a[pos] * b_val[p] : V();
            else cv[u] = V();
        }
        f(cj, cv);
    }
    wave_sync();   // the chunk arrays may be rewritten now
}

// One wave handles the 64 segments (p0, len, a) its lanes hold: the long ones are walked 64-wide
// by the whole wave, one after the other, the rest is flattened.
template <bool HAS_VAL, typename V, typename F>
__device__ __forceinline__ void wave_chunk(FlatChunk<V, WAVE> &c, int64_t p0, int64_t len, V a,
                                           const int32_t *__restrict__ b_col, const V *__restrict__ b_val, F &f)
{
    const bool is_long = len >= T_LONG;
    unsigned long long m = __ballot(is_long);
    while (m) {
        const int src = __ffsll((long long)m) - 1;
        m &= m - 1ull;
        const int64_t sp0 = __shfl(p0, src, WAVE);
        const int64_t slen = __shfl(len, src, WAVE);
        V sa = V();
        if constexpr (HAS_VAL) sa = __shfl(a, src, WAVE);
        exec_segment<WAVE, FLAT_U, HAS_VAL>(b_col, b_val, sp0, slen, lane_id(), sa, f);
    }
    group_flat<WAVE, HAS_VAL>(c, p0, is_long ? 0u : (uint32_t)len, a, b_col, b_val, f);
}

// Wave version: the 64 lanes of one wave walk one row; no workgroup barrier.
template <bool HAS_VAL, typename V, typename SegFn, typename F>
__device__ __forceinline__ void wave_traverse(const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                                              int64_t e0, int64_t e1, SegFn seg, const int32_t *__restrict__ b_col,
                                              const V *__restrict__ b_val, FlatChunk<V, WAVE> &c, F f)
{
    const int lane = lane_id();
    for (int64_t base = e0; base < e1; base += WAVE) {
        const int64_t e = base + lane;
        int64_t p0 = 0, len = 0;
        V a = V();
        if (e < e1) {
            const int32_t k = a_col[e];
            if constexpr (HAS_VAL) a = a_val[e];
            seg(k, p0, len);
        }
        wave_chunk<HAS_VAL>(c, p0, len, a, b_col, b_val, f);
    }
}

// LDS scratch of a workgroup-wide flattened chunk of up to THREADS entries.  RPT: products per thread up to which
// the entries of a chunk are found by rank (below); the mark bitmap grows with it.
template <typename V, int THREADS, int RPT = 16>
struct WgChunk {
    static constexpr uint32_t RANK_CAP = (uint32_t)RPT * THREADS;   // most products of a chunk whose entries are found by rank
    static constexpr int START_WORDS = THREADS * RPT / 32 + 32;
    uint32_t excl[THREADS + 1];
    long long pbase[THREADS];
    V a[THREADS];
    union alignas(8) {
        uint16_t first[THREADS + 2];       // entry of the first product of every block of 2^bshift products
        uint32_t start[START_WORDS];       // bit q set: a segment starts at product q (RANK_CAP bits + padding for batches of up to 16 per lane)
    };
    uint32_t wsum[THREADS / WAVE];
    uint32_t wcnt[THREADS / WAVE];
    uint32_t wsumr[THREADS / WAVE];        // (runs) per-wave sums of the lengths rounded up to whole runs
    uint32_t next;                         // (runs) first product slot of the next batch nobody has taken yet
    unsigned long long alloc;              // (wg_flat_chunk_keep) products (low word) and non-empty segments handed out so far
};

// The whole workgroup flattens the `nent` (1..THREADS) segments held by its first nent threads
// (p0, len, a; len = 0 in the other threads): the products of the concatenation are dealt out
// evenly to the waves whatever the lengths of the single segments, so a row with three entries
// that point to long rows of B keeps every wave as busy as a row with a thousand short ones.
// Every wave takes one contiguous span of the products, 256 at a time.  The entry a product
// belongs to is found in one of two ways:
//   * a chunk of at most RPT (16, or what the chunk type says) products per thread marks the first product of every non-empty
//     segment in a bitmap; the entry of product q (counting non-empty entries only, which are
//     stored compacted) is the number of marks at or before q, minus one: one broadcast read of
//     the 64 marks of the wave's batch and a population count, on top of a running count that the
//     wave carries along its span;
//   * a larger chunk (long segments) uses a binary search over the prefix sums, narrowed
//     beforehand to the few entries a batch of 256 can touch: a table built once per chunk gives
//     the entry of the first product of every block of products.  The searches of a batch have
//     the same, wave-uniform number of steps and run interleaved.  Without values (the symbolic
//     pass) such a chunk is walked in runs of WU consecutive column ids per lane instead, its
//     batches handed out from a counter rather than in equal spans (see there).
// WU is the number of products per lane and batch.  The products of one chunk must number less
// than 2^31.
// Every thread calls it; the chunk arrays must be free on entry (the call ends with a barrier).
// Returns the number of products of the chunk.
template <int THREADS, bool HAS_VAL, int WU = FLAT_U, typename V, typename F, int RPT>
__device__ __forceinline__ uint32_t wg_flat_chunk(WgChunk<V, THREADS, RPT> &c, int nent, int64_t p0, uint32_t len, V a,
                                              const int32_t *__restrict__ b_col, const V *__restrict__ b_val, F &f)
{
    constexpr int NW = THREADS / WAVE;
    constexpr uint32_t RANK_CAP = WgChunk<V, THREADS, RPT>::RANK_CAP;
    constexpr int START_WORDS = WgChunk<V, THREADS, RPT>::START_WORDS;
    static_assert(THREADS <= 1024, "entry ids are kept in 16 bits and one block table entry per thread");
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1), wave = tid / WAVE;
    for (int j = tid; j < START_WORDS; j += THREADS) c.start[j] = 0u;
    uint32_t incl = wave_inclusive_scan_u32(len);
    // non-empty segments are numbered on their own
    const unsigned long long live = __ballot(len > 0);
    if (lane == WAVE - 1) { c.wsum[wave] = incl; c.wcnt[wave] = (uint32_t)__popcll(live); }
    // column ids only: the same sums over the lengths rounded up to whole runs of WU (see below)
    constexpr bool RUNS = !HAS_VAL && WU % 4 == 0;
    const uint32_t lenr = (len + (uint32_t)(WU - 1)) & ~(uint32_t)(WU - 1);
    uint32_t inclr = 0;
    if constexpr (RUNS) {
        inclr = wave_inclusive_scan_u32(lenr);
        if (lane == WAVE - 1) c.wsumr[wave] = inclr;
    }
    __syncthreads();
    uint32_t total, ctotal;
    const uint32_t before = waves_before_u32<NW>(c.wsum, wave, total);
    const uint32_t cbefore = waves_before_u32<NW>(c.wcnt, wave, ctotal);
    incl += before;
    if (total == 0) {   // uniform
        __syncthreads();
        return 0;
    }
    const uint32_t span = ((total + NW - 1) / NW + (WAVE - 1)) & ~(uint32_t)(WAVE - 1);
    const uint32_t qs = (uint32_t)wave * span;
    const uint32_t qe = qs + span < total ? qs + span : total;
    int32_t cj[WU];
    V cb[WU];   // values of B
    int cp[WU];
    // Runs (column ids only, below) pay when the segments are at least a run long on average - shorter ones leave
    // most of a run's slots empty (rows of B of 8 entries in runs of 16: 0.93 against 0.60 ms on a test input, rows
    // of 24: 0.86 against 1.62 ms) - and long runs are worth more than the marks even for a small chunk (R-MAT,
    // 16 ids per run: 15.7 against 15.9 ms), short ones are not (rect, 4 ids per run: 0.78 against 0.68 ms).
    const bool use_runs = RUNS && (unsigned long long)total >= (unsigned long long)ctotal * (unsigned)WU &&
                          (WU >= 8 || total > RANK_CAP);   // uniform
    if constexpr (RUNS && WU > 4) {
        // (a chunk of short segments: the same with four column ids per lane and batch - the marks, runs of four
        // or the search, whichever applies - which also keeps the registers of those paths out of this one)
        if (!use_runs) {   // uniform
            __syncthreads();   // (everyone has read the waves' sums)
            return wg_flat_chunk<THREADS, HAS_VAL, 4>(c, nent, p0, len, a, b_col, b_val, f);
        }
    }
    if (!use_runs && total <= RANK_CAP) {   // uniform
        const uint32_t ex = incl - len;
        if (len > 0) {
            const uint32_t ce = cbefore + __builtin_amdgcn_mbcnt_hi((uint32_t)(live >> 32),
                                                                    __builtin_amdgcn_mbcnt_lo((uint32_t)live, 0u));
            c.pbase[ce] = (long long)p0 - (long long)ex;
            c.a[ce] = a;
            atomicOr(&c.start[ex >> 5], 1u << (ex & 31u));
        }
        __syncthreads();
        if (qs < total) {   // uniform for the wave
            const unsigned long long *marks = reinterpret_cast<const unsigned long long *>(c.start);
            // segments that start before the wave's span
            uint32_t run = 0;
            for (uint32_t j = (uint32_t)lane; j < (qs >> 6); j += WAVE) run += (uint32_t)__popcll(marks[j]);
            run = wave_sum_u32(run);
            const unsigned long long upto = (2ull << lane) - 1ull;   // this lane's product and those before it
            for (uint32_t q0 = qs; q0 < qe; q0 += WAVE * WU) {
                // Every stage of a batch is straight-line code over its WU products, with
                // unconditional reads (a lane past the end of the span reads product 0, which exists), so
                // that the reads of one stage are in flight together.
                unsigned long long m[WU];
#pragma unroll
                for (int u = 0; u < WU; ++u) m[u] = marks[(q0 >> 6) + u];   // one address for the wave
                bool ok[WU];
                uint32_t qq[WU];
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    const uint32_t q = q0 + u * WAVE + lane;
                    ok[u] = q < qe;
                    const uint32_t rank = run + (uint32_t)__popcll(m[u] & upto);   // >= 1: product 0 starts a segment
                    run += (uint32_t)__popcll(m[u]);
                    cp[u] = ok[u] ? (int)rank - 1 : 0;
                    qq[u] = ok[u] ? q : 0u;
                }
                long long pb[WU];
                V av[WU];
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    pb[u] = c.pbase[cp[u]];
                    if constexpr (HAS_VAL) av[u] = c.a[cp[u]];
                }
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    const int64_t p = pb[u] + (long long)qq[u];
                    cj[u] = ok[u] ? b_col[p] : -1;
                    if constexpr (HAS_VAL) cb[u] = ok[u] ? b_val[p] : V();
                }
                V cv[WU];
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    if constexpr (HAS_VAL) cv[u] = av[u] * cb[u];
                    else cv[u] = V();
                }
                if constexpr (std::is_invocable_v<F &, int32_t(&)[WU], V(&)[WU], uint32_t>) f(cj, cv, q0);
                else f(cj, cv);
            }
        }
        __syncthreads();
        return total;
    }
    if constexpr (RUNS) if (use_runs) {
        // Column ids only (the symbolic pass: whole rows of B, mostly long ones, and a set of columns as the
        // result, so that a column seen twice does no harm).  Every lane takes a run of WU consecutive entries
        // of ONE segment with 16-byte loads: the segments are laid out with their lengths rounded up to whole
        // runs, so no run straddles two segments; the last run of a segment is moved back to end with the
        // segment (it repeats entries of the run before), and a lane past the end of the chunk repeats the last
        // run.  Only a segment shorter than one run needs loads of single entries.  One search per lane and
        // batch finds the segment; excl[e + 1] carries in its low bits by how much segment e was rounded up.
        uint32_t totalr;
        inclr += waves_before_u32<NW>(c.wsumr, wave, totalr);
        if (tid < nent) {
            c.excl[tid + 1] = inclr | (lenr - len);
            c.pbase[tid] = (long long)p0 - (long long)(inclr - lenr);
        }
        if (tid == 0) {
            c.excl[0] = 0u;
            c.next = 0u;
        }
        __syncthreads();
        constexpr uint32_t LOW = (uint32_t)(WU - 1);
        int bshift = 8;
        while (((totalr - 1) >> bshift) >= (uint32_t)(THREADS - 1)) ++bshift;
        const int nblk = (int)((totalr - 1) >> bshift) + 1;
        const int top = nent > 1 ? 1 << (31 - __clz(nent - 1)) : 0;
        if (tid <= nblk) {
            int pos = nent - 1;
            if (tid < nblk) {
                const uint32_t q = ((uint32_t)tid << bshift) | LOW;
                pos = 0;
                for (int step = top; step > 0; step >>= 1) {
                    const int t = pos + step;
                    const uint32_t ex = c.excl[t < nent ? t : nent - 1];
                    pos = (t < nent && ex <= q) ? t : pos;   // last entry starting at or before q (skips empty ones)
                }
            }
            c.first[tid] = (uint16_t)pos;
        }
        __syncthreads();
        // Batches are handed out one at a time from a counter in LDS, the ticket of the next one being drawn
        // before the current one is worked on: batches differ in cost (searches are longer where segments are
        // short, and the short segments of a chunk sit together, the entries of a row of A being in column
        // order), so equal shares of the products would not be equal shares of the time.
        auto draw = [&]() {
            uint32_t t = 0u;
            if (lane == 0) t = atomicAdd(&c.next, (uint32_t)(WAVE * WU));
            return t;
        };
        uint32_t ticket = draw();
        for (;;) {
            const uint32_t q0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)ticket);
            if (q0 >= totalr) break;   // uniform
            ticket = draw();
            const uint32_t qlast = q0 + WAVE * WU - 1 < totalr - 1 ? q0 + WAVE * WU - 1 : totalr - 1;
            const int lo = c.first[q0 >> bshift];
            const int hi = c.first[(qlast >> bshift) + 1];   // the entry of a later run, or the last entry
            const int width = __builtin_amdgcn_readfirstlane(hi - lo);
            uint32_t q = q0 + (uint32_t)lane * WU;
            q = q < totalr ? q : totalr - (uint32_t)WU;   // (q0 <= totalr - WU: both are multiples of WU)
            const uint32_t key = q | LOW;
            int fp = lo;
            for (int step = width > 0 ? 1 << (31 - __clz(width)) : 0; step > 0; step >>= 1) {
                const int t = fp + step;
                const uint32_t ex = c.excl[t <= hi ? t : hi];
                fp = (t <= hi && ex <= key) ? t : fp;
            }
            const uint32_t endw = c.excl[fp + 1];
            const uint32_t begin = c.excl[fp] & ~LOW;
            const long long pb = c.pbase[fp];
            const uint32_t nvalid = (endw & ~LOW) - (endw & LOW) - q;   // entries of the segment from q on: >= 1
            const bool tail = nvalid < (uint32_t)WU;
            const bool tiny = tail && q == begin;   // the whole segment is shorter than a run
            const uint32_t back = tail && !tiny ? (uint32_t)WU - nvalid : 0u;
            const int32_t *src = b_col + (pb + (long long)q - (long long)back);
            V cv[WU] = {};
            if (__ballot(tiny) == 0ull) {   // uniform
                const Int4U *src4 = reinterpret_cast<const Int4U *>(src);
#pragma unroll
                for (int g = 0; g < WU / 4; ++g) {
                    const Int4U x = src4[g];
#pragma unroll
                    for (int i = 0; i < 4; ++i) cj[g * 4 + i] = x.v[i];
                }
                if constexpr (std::is_invocable_v<F &, int32_t(&)[WU], V(&)[WU], AllValid>) f(cj, cv, AllValid{});
                else f(cj, cv);
            } else {
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    cj[u] = -1;
                    if (!tiny || (uint32_t)u < nvalid) cj[u] = src[u];
                }
                f(cj, cv);
            }
        }
        __syncthreads();
        return total;
    }
    if (tid < nent) {
        c.excl[tid] = incl - len;
        c.pbase[tid] = (long long)p0 - (long long)(incl - len);
        c.a[tid] = a;
    }
    __syncthreads();
    // blocks of 2^bshift products, at least 256 products each and fewer than THREADS of them
    int bshift = 8;
    while (((total - 1) >> bshift) >= (uint32_t)(THREADS - 1)) ++bshift;
    const int nblk = (int)((total - 1) >> bshift) + 1;
    const int top = nent > 1 ? 1 << (31 - __clz(nent - 1)) : 0;
    if (tid <= nblk) {
        int pos = nent - 1;
        if (tid < nblk) {
            const uint32_t q = (uint32_t)tid << bshift;
            pos = 0;
            for (int step = top; step > 0; step >>= 1) {
                const int t = pos + step;
                const uint32_t ex = c.excl[t < nent ? t : nent - 1];   // unconditional read: no branch around it
                pos = (t < nent && ex <= q) ? t : pos;   // last entry starting at or before q (skips empty ones)
            }
        }
        c.first[tid] = (uint16_t)pos;
    }
    __syncthreads();
    if (qs < total) {   // uniform for the wave
        auto fetch = [&](uint32_t q0, int32_t (&fj)[WU], V (&fb)[WU], int (&fp)[WU]) {
            const uint32_t qlast = q0 + WAVE * WU - 1 < qe - 1 ? q0 + WAVE * WU - 1 : qe - 1;
            const int lo = c.first[q0 >> bshift];
            const int hi = c.first[(qlast >> bshift) + 1];   // the entry of a later product, or the last entry
            const int width = __builtin_amdgcn_readfirstlane(hi - lo);
#pragma unroll
            for (int u = 0; u < WU; ++u) fp[u] = lo;
            if (!HAS_VAL && width == 0) {
                // symbolic pass (whole rows of B, often long): the batch lies in one row of B, no search,
                // one read of the segment's base
                const long long base = c.pbase[lo];
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    const uint32_t q = q0 + u * WAVE + lane;
                    const bool ok = q < qe;
                    const int64_t p = base + (long long)q;
                    fj[u] = ok ? b_col[p] : -1;
                    if constexpr (HAS_VAL) fb[u] = ok ? b_val[p] : V();
                    else fb[u] = V();
                }
                return;
            }
            for (int step = width > 0 ? 1 << (31 - __clz(width)) : 0; step > 0; step >>= 1) {
                // the reads of one step are unconditional (index clamped) so that they are issued together
                int t[WU];
                uint32_t ex[WU];
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    t[u] = fp[u] + step;
                    ex[u] = c.excl[t[u] <= hi ? t[u] : hi];
                }
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    const uint32_t q = q0 + u * WAVE + lane;
                    fp[u] = (t[u] <= hi && ex[u] <= q) ? t[u] : fp[u];
                }
            }
            long long pb[WU];
#pragma unroll
            for (int u = 0; u < WU; ++u) pb[u] = c.pbase[fp[u]];   // (reads of LDS together, ahead of the loads)
#pragma unroll
            for (int u = 0; u < WU; ++u) {
                const uint32_t q = q0 + u * WAVE + lane;
                const bool ok = q < qe;
                const int64_t p = pb[u] + (long long)q;
                fj[u] = ok ? b_col[p] : -1;
                if constexpr (HAS_VAL) fb[u] = ok ? b_val[p] : V();
                else fb[u] = V();
            }
        };
        for (uint32_t q0 = qs; q0 < qe; q0 += WAVE * WU) {
            fetch(q0, cj, cb, cp);
            V cv[WU];
#pragma unroll
            for (int u = 0; u < WU; ++u) {
                if constexpr (HAS_VAL) cv[u] = c.a[cp[u]] * cb[u];
                else cv[u] = V();
            }
            // an accumulator may ask for the number of the batch's first product inside the chunk: the
            // product of lane l, position u is number q0 + u*64 + l
            if constexpr (std::is_invocable_v<F &, int32_t(&)[WU], V(&)[WU], uint32_t>) f(cj, cv, q0);
            else f(cj, cv);
        }
    }
    __syncthreads();
    return total;
}

// The same flattening for a chunk whose products the caller keeps: every thread ends up with its
// share of the products (column id, a*b) in registers, kc[i] < 0 where it has none, and mark(col)
// has been called once per product.  Needs at most NB * FLAT_U products per thread
// (total <= NB * FLAT_U * THREADS) and total <= WgChunk::RANK_CAP; otherwise nothing is fetched and
// fits = false.  The segments are laid end to end wave by wave, in the order in which the waves draw their share
// of the product numbers from a counter in LDS (the order of the products of a chunk means nothing), which spares
// the barrier and the scan over the waves' sums that a fixed order would need.  clean: the marks and the counter
// are as this function leaves them (all zero); after any other use of the chunk pass false and they are cleared
// first.  Every thread calls it; ends with a barrier; returns the number of products.
template <int THREADS, int NB, typename V, typename M, int RPT>
__device__ __forceinline__ uint32_t wg_flat_chunk_keep(WgChunk<V, THREADS, RPT> &c, int /*nent*/, int64_t p0, uint32_t len, V a,
                                                   const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
                                                   int32_t (&kc)[NB * FLAT_U], V (&kv)[NB * FLAT_U], M &mark,
                                                   bool &fits, bool clean)
{
    constexpr int NW = THREADS / WAVE;
    constexpr uint32_t RANK_CAP = WgChunk<V, THREADS, RPT>::RANK_CAP;
    constexpr int START_WORDS = WgChunk<V, THREADS, RPT>::START_WORDS;
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1), wave = tid / WAVE;
    if (!clean) {   // uniform
        for (int j = tid; j < START_WORDS; j += THREADS) c.start[j] = 0u;
        if (tid == 0) c.alloc = 0ull;
        __syncthreads();
    }
    uint32_t incl = wave_inclusive_scan_u32(len);
    const unsigned long long live = __ballot(len > 0);
    unsigned long long got = 0ull;
    if (lane == WAVE - 1) got = atomicAdd(&c.alloc, (unsigned long long)incl | ((unsigned long long)__popcll(live) << 32));
#pragma unroll
    for (int i = 0; i < NB * FLAT_U; ++i) { kc[i] = -1; kv[i] = V(); }
    const uint32_t before = wave_read_lane_u32((uint32_t)got, WAVE - 1);
    const uint32_t cbefore = wave_read_lane_u32((uint32_t)(got >> 32), WAVE - 1);
    incl += before;
    const uint32_t ex = incl - len;
    if (len > 0 && incl <= RANK_CAP) {   // (beyond the marks nothing is fetched anyway, see fits)
        const uint32_t ce = cbefore + __builtin_amdgcn_mbcnt_hi((uint32_t)(live >> 32),
                                                                __builtin_amdgcn_mbcnt_lo((uint32_t)live, 0u));
        c.pbase[ce] = (long long)p0 - (long long)ex;
        c.a[ce] = a;
        atomicOr(&c.start[ex >> 5], 1u << (ex & 31u));
    }
    __syncthreads();
    const uint32_t total = (uint32_t)c.alloc;
    fits = total <= RANK_CAP && total <= (uint32_t)(NB * FLAT_U * THREADS);
    if (total == 0 || !fits) {   // uniform
        __syncthreads();
        for (int j = tid; j < START_WORDS; j += THREADS) c.start[j] = 0u;
        if (tid == 0) c.alloc = 0ull;
        return total;
    }
    const uint32_t span = ((total + NW - 1) / NW + (WAVE - 1)) & ~(uint32_t)(WAVE - 1);   // <= NB * FLAT_U * WAVE
    const uint32_t qs = (uint32_t)wave * span;
    const uint32_t qe = qs + span < total ? qs + span : total;
    if (qs < total) {   // uniform for the wave
        const unsigned long long *marks = reinterpret_cast<const unsigned long long *>(c.start);
        uint32_t run = 0;
        for (uint32_t j = (uint32_t)lane; j < (qs >> 6); j += WAVE) run += (uint32_t)__popcll(marks[j]);
        run = wave_sum_u32(run);
        const unsigned long long upto = (2ull << lane) - 1ull;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const uint32_t q0 = qs + (uint32_t)b * WAVE * FLAT_U;
            if (q0 < qe) {   // uniform for the wave
                unsigned long long m[FLAT_U];
#pragma unroll
                for (int u = 0; u < FLAT_U; ++u) m[u] = marks[(q0 >> 6) + u];
                bool ok[FLAT_U];
                int cp[FLAT_U];
#pragma unroll
                for (int u = 0; u < FLAT_U; ++u) {
                    const uint32_t q = q0 + u * WAVE + lane;
                    ok[u] = q < qe;
                    const uint32_t rank = run + (uint32_t)__popcll(m[u] & upto);
                    run += (uint32_t)__popcll(m[u]);
                    cp[u] = ok[u] ? (int)rank - 1 : 0;
                }
                long long pb[FLAT_U];
                V av[FLAT_U];
#pragma unroll
                for (int u = 0; u < FLAT_U; ++u) {
                    pb[u] = c.pbase[cp[u]];
                    av[u] = c.a[cp[u]];
                }
                V cb[FLAT_U];
#pragma unroll
                for (int u = 0; u < FLAT_U; ++u) {
                    const int64_t p = pb[u] + (long long)(q0 + u * WAVE + lane);
                    kc[b * FLAT_U + u] = ok[u] ? b_col[p] : -1;
                    cb[u] = ok[u] ? b_val[p] : V();
                }
#pragma unroll
                for (int u = 0; u < FLAT_U; ++u) {
                    kv[b * FLAT_U + u] = av[u] * cb[u];
                    if (kc[b * FLAT_U + u] >= 0) mark(kc[b * FLAT_U + u]);
                }
            }
        }
    }
    __syncthreads();
    // (left clean for the next call; whatever the caller does next has a barrier before the chunk is used again)
    for (int j = tid; j < (int)((total >> 5) + 2u) && j < START_WORDS; j += THREADS) c.start[j] = 0u;
    if (tid == 0) c.alloc = 0ull;
    return total;
}

// Workgroup version of the row traversal: chunks of THREADS entries of A, each flattened over the
// whole workgroup.  Every thread of the (1-D) workgroup must call it.  seg(k, p0, len) gives the
// segment of B's arrays that entry k expands to.  Ends with a barrier.
template <int THREADS, bool HAS_VAL, int WU = FLAT_U, typename V, typename SegFn, typename F, int RPT>
__device__ __forceinline__ void wg_traverse(const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                                            int64_t e0, int64_t e1, SegFn seg, const int32_t *__restrict__ b_col,
                                            const V *__restrict__ b_val, WgChunk<V, THREADS, RPT> &c, F f)
{
    const int tid = threadIdx.x;
    for (int64_t base = e0; base < e1; base += THREADS) {
        const int64_t e = base + tid;
        int64_t p0 = 0, len = 0;
        V a = V();
        if (e < e1) {
            const int32_t k = a_col[e];
            if constexpr (HAS_VAL) a = a_val[e];
            seg(k, p0, len);
        }
        const int64_t left = e1 - base;
        wg_flat_chunk<THREADS, HAS_VAL, WU>(c, left < THREADS ? (int)left : THREADS, p0, (uint32_t)len, a, b_col, b_val, f);
    }
}

}  // namespace ocean
