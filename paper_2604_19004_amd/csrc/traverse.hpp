// Traversal of the intermediate products of one row of C = A*B (Gustavson's two
// nested loops, paper Section 2.1) by a whole workgroup, one wave or a group
// of lanes.
//
// The kernels are bound by instruction issue and by dependent-access latency,
// not by bandwidth, so what matters is that all 64 lanes of a wave carry a
// product in every instruction and that independent memory operations are in
// flight together.  Rows of B referenced by one row of A differ wildly in
// length on power-law matrices; a fixed "lanes per row of B" mapping leaves
// most lanes idle.  Therefore:
//   * entries A_ik whose row of B is shorter than T_LONG are FLATTENED: a wave
//     takes 64 entries, prefix-sums their lengths, and lane l then handles
//     products l, l+64, ... of the concatenated segments, finding the entry of
//     a product by a 6-step search over the prefix sums kept in LDS;
//   * longer rows of B are walked 64-wide by a whole wave (coalesced), queued
//     in LDS first so that the waves of a workgroup share them evenly, and the
//     very long ones (>= 4*THREADS) by the whole workgroup.
// Products reach the accumulator in batches: f(cj, cv) receives U column ids
// (negative = none) and values a*b per lane, so that the accumulator's own
// dependent LDS round trips (hash probes) overlap across the batch.
#pragma once

#include "ocean_internal.hpp"

namespace ocean {

constexpr int T_LONG = 128;
constexpr int FLAT_U = 4;
constexpr int MAX_HUGE = 8;

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

// G lanes (a power of two <= 64, consecutive lanes of one wave) flatten the G
// segments (p0, len, a) they hold, len < 2^24.  Every lane of the group calls it.
// Several waves may flatten the same chunk (each with its own FlatChunk copy)
// and share its batches: this one takes batches first, first+stride, ...
template <int G, bool HAS_VAL, typename V, typename F>
__device__ __forceinline__ void group_flat(FlatChunk<V, G> &c, int64_t p0, uint32_t len, V a,
                                           const int32_t *__restrict__ b_col, const V *__restrict__ b_val, F &f,
                                           uint32_t first = 0, uint32_t stride = 1)
{
    const int sub = lane_id() & (G - 1);
    uint32_t incl = len;
#pragma unroll
    for (int off = 1; off < G; off <<= 1) {
        const uint32_t o = __shfl_up(incl, off, G);
        if (sub >= off) incl += o;
    }
    const uint32_t total = __shfl(incl, G - 1, G);
    if (G == WAVE && total == 0) return;   // uniform for a whole wave
    c.excl[sub] = incl - len;
    c.pbase[sub] = (long long)p0 - (long long)(incl - len);
    c.a[sub] = a;
    wave_sync();
    for (uint32_t q0 = first * (G * FLAT_U); q0 < total; q0 += stride * (G * FLAT_U)) {
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

// Queue of the long segments of a row, shared by the waves of a workgroup.
template <typename V, int CAP>
struct LongQueue {
    unsigned long long p0[CAP];
    int32_t len[CAP];          // negative: registered as huge
    V a[CAP];
    int32_t huge[MAX_HUGE];
    unsigned int n;            // running counters: they only grow while a row is processed
    unsigned int n_huge;
};

// Values of the queue's running counters when the queue was last drained, kept
// in registers by every thread.  Reset it together with q.n / q.n_huge; carry
// it over when the same row is traversed again (one call per column window).
struct TravState {
    unsigned start = 0, hstart = 0;
};

// Queue one long segment.  False when the queue is full: the caller walks it itself.
template <int THREADS, typename V, int CAP>
__device__ __forceinline__ bool queue_push(LongQueue<V, CAP> &q, const TravState &st, int64_t p0, int64_t len, V a)
{
    constexpr int T_HUGE = 4 * THREADS;
    const unsigned idx = atomicAdd(&q.n, 1u) - st.start;
    if (idx >= (unsigned)CAP) return false;
    q.p0[idx] = (unsigned long long)p0;
    q.a[idx] = a;
    int32_t l32 = (int32_t)len;
    if (len >= T_HUGE) {
        const unsigned h = atomicAdd(&q.n_huge, 1u) - st.hstart;
        if (h < (unsigned)MAX_HUGE) { q.huge[h] = (int32_t)idx; l32 = -l32; }
    }
    q.len[idx] = l32;
    return true;
}

// Walk everything queued since st (all pushes must be visible: barrier before) and advance st.
// Every thread of the workgroup calls it; no barrier inside.
template <int THREADS, bool HAS_VAL, typename V, int CAP, typename F>
__device__ __forceinline__ void queue_drain(LongQueue<V, CAP> &q, TravState &st, const int32_t *__restrict__ b_col,
                                            const V *__restrict__ b_val, F &f)
{
    constexpr int NW = THREADS / WAVE;
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1), wave = tid / WAVE;
    const unsigned total = q.n - st.start;
    const unsigned htotal = q.n_huge - st.hstart;
    const int nq = (int)(total < (unsigned)CAP ? total : (unsigned)CAP);
    const int nh = (int)(htotal < (unsigned)MAX_HUGE ? htotal : (unsigned)MAX_HUGE);
    for (int i = wave; i < nq; i += NW) {
        const int32_t len = q.len[i];
        if (len > 0) exec_segment<WAVE, FLAT_U, HAS_VAL>(b_col, b_val, (int64_t)q.p0[i], len, lane, q.a[i], f);
    }
    for (int h = 0; h < nh; ++h) {
        const int i = q.huge[h];
        exec_segment<THREADS, FLAT_U, HAS_VAL>(b_col, b_val, (int64_t)q.p0[i], -(int64_t)q.len[i], tid, q.a[i], f);
    }
    st.start += total;
    st.hstart += htotal;
}

// One wave handles the 64 segments (p0, len, a) its lanes hold: the long ones go to the queue (or
// are walked right away by the whole wave when there is no queue / it is full), the rest is flattened.
// With stride > 1 the same 64 segments are given to `stride` waves, which share the flattened part
// (this wave takes batches first, first+stride, ...); only the wave with first == 0 handles the long ones.
template <int THREADS, bool HAS_VAL, typename V, int CAP, typename F>
__device__ __forceinline__ void wave_chunk(FlatChunk<V, WAVE> &c, LongQueue<V, CAP> *q, const TravState &st, int64_t p0,
                                           int64_t len, V a, const int32_t *__restrict__ b_col,
                                           const V *__restrict__ b_val, F &f, uint32_t first = 0, uint32_t stride = 1)
{
    const bool is_long = len >= T_LONG;
    bool pushed = false;
    if (is_long && q != nullptr && first == 0) pushed = queue_push<THREADS>(*q, st, p0, len, a);
    unsigned long long m = __ballot(is_long && !pushed && first == 0);
    while (m) {
        const int src = __ffsll((long long)m) - 1;
        m &= m - 1ull;
        const int64_t sp0 = __shfl(p0, src, WAVE);
        const int64_t slen = __shfl(len, src, WAVE);
        V sa = V();
        if constexpr (HAS_VAL) sa = __shfl(a, src, WAVE);
        exec_segment<WAVE, FLAT_U, HAS_VAL>(b_col, b_val, sp0, slen, lane_id(), sa, f);
    }
    group_flat<WAVE, HAS_VAL>(c, p0, is_long ? 0u : (uint32_t)len, a, b_col, b_val, f, first, stride);
}

// Workgroup version.  Every thread of the (1-D) workgroup must call it.  q.n
// and q.n_huge must be visible (barrier) on entry and equal to st (zero after a
// reset).  seg(k, p0, len) gives the segment of B's arrays that entry k expands
// to.  chunks: one FlatChunk per wave.  Ends with a barrier.
template <int THREADS, bool HAS_VAL, typename V, int CAP, typename SegFn, typename F>
__device__ __forceinline__ void wg_traverse(const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                                            int64_t e0, int64_t e1, SegFn seg, const int32_t *__restrict__ b_col,
                                            const V *__restrict__ b_val, FlatChunk<V, WAVE> *chunks,
                                            LongQueue<V, CAP> &q, TravState &st, F f)
{
    constexpr int NW = THREADS / WAVE;
    const int tid = threadIdx.x;
    const int wave = tid / WAVE;
    // A row with many entries: every wave takes its own chunks of 64 entries.  A row with few: all
    // waves read the same chunks and share the products of each.  No barrier inside either loop.
    const bool shared = (e1 - e0) < (int64_t)WAVE * NW / 2;
    const int64_t first_base = shared ? e0 : e0 + (int64_t)wave * WAVE;
    const int64_t base_step = shared ? WAVE : THREADS;
    for (int64_t base = first_base; base < e1; base += base_step) {
        const int64_t e = base + (tid & (WAVE - 1));
        int64_t p0 = 0, len = 0;
        V a = V();
        if (e < e1) {
            const int32_t k = a_col[e];
            if constexpr (HAS_VAL) a = a_val[e];
            seg(k, p0, len);
        }
        wave_chunk<THREADS, HAS_VAL>(chunks[wave], &q, st, p0, len, a, b_col, b_val, f, shared ? (uint32_t)wave : 0u,
                                     shared ? (uint32_t)NW : 1u);
    }
    __syncthreads();
    queue_drain<THREADS, HAS_VAL>(q, st, b_col, b_val, f);
    __syncthreads();
}

// Wave version: the 64 lanes of one wave walk one row; no workgroup barrier, no queue.
template <bool HAS_VAL, typename V, typename SegFn, typename F>
__device__ __forceinline__ void wave_traverse(const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                                              int64_t e0, int64_t e1, SegFn seg, const int32_t *__restrict__ b_col,
                                              const V *__restrict__ b_val, FlatChunk<V, WAVE> &c, F f)
{
    const int lane = lane_id();
    const TravState st;
    for (int64_t base = e0; base < e1; base += WAVE) {
        const int64_t e = base + lane;
        int64_t p0 = 0, len = 0;
        V a = V();
        if (e < e1) {
            const int32_t k = a_col[e];
            if constexpr (HAS_VAL) a = a_val[e];
            seg(k, p0, len);
        }
        wave_chunk<WAVE, HAS_VAL>(c, static_cast<LongQueue<V, 1> *>(nullptr), st, p0, len, a, b_col, b_val, f);
    }
}

}  // namespace ocean
