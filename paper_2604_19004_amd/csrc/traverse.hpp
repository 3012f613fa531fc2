// Traversal of the intermediate products of one row of C = A*B (Gustavson's two
// nested loops, paper Section 2.1) by a whole workgroup or by one wave.
//
// Rows of B referenced by one row of A differ wildly in length on power-law
// matrices, so a fixed "lanes per row of B" mapping leaves most of a 64-wide
// wave idle.  Every entry A_ik is therefore classified by the length of the
// segment of B it expands to:
//     short   (< T_MED)    walked by the lane that loaded the entry
//     medium  (< T_LONG)   queued in LDS, then walked by a 16-lane group
//     long                 queued, walked by a whole wave (coalesced 64-wide)
//     huge    (>= 4*THREADS, workgroup version only) walked by the whole workgroup
// f(col, value) is called once per product; queues live in LDS.
#pragma once

#include "ocean_internal.hpp"

namespace ocean {

constexpr int T_MED = 8;
constexpr int T_LONG = 128;
constexpr int MED_LANES = 16;
constexpr int MAX_HUGE = 8;

template <typename V, int CAP>
struct TravQueue {
    unsigned long long p0[CAP];
    int32_t len[CAP];          // negative: registered as huge
    V a[CAP];
    int32_t huge[MAX_HUGE];
    unsigned int n;            // running counters: they only grow while a row is processed
    unsigned int n_huge;
};

// Values of the queue's running counters at the start of the next chunk, kept
// in registers by every thread.  Reset it together with q.n / q.n_huge; carry
// it over when the same row is traversed again (one call per column window).
struct TravState {
    unsigned start = 0, hstart = 0;
};

// Workgroup version.  Every thread of the (1-D) workgroup must call it.  q.n
// and q.n_huge must be visible (barrier) on entry and equal to st (zero after a
// reset).  seg(k, p0, len) gives the segment of B's arrays that entry k expands
// to; f(col, value) is called once per product.
template <int THREADS, bool HAS_VAL, typename V, int CAP, typename SegFn, typename F>
__device__ __forceinline__ void wg_traverse(const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                                            int64_t e0, int64_t e1, SegFn seg, const int32_t *__restrict__ b_col,
                                            const V *__restrict__ b_val, TravQueue<V, CAP> &q, TravState &st, F f)
{
    constexpr int NW = THREADS / WAVE;
    constexpr int NG = THREADS / MED_LANES;
    constexpr int T_HUGE = 4 * THREADS;
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1), wave = tid / WAVE;
    const int gl = tid & (MED_LANES - 1), grp = tid / MED_LANES;
    unsigned start = st.start, hstart = st.hstart;
    for (int64_t base = e0; base < e1; base += THREADS) {
        const int64_t e = base + tid;
        if (e < e1) {
            const int32_t k = a_col[e];
            V a = V();
            if constexpr (HAS_VAL) a = a_val[e];
            int64_t p0, len;
            seg(k, p0, len);
            bool queued = false;
            if (len >= T_MED) {
                const unsigned idx = atomicAdd(&q.n, 1u) - start;
                if (idx < (unsigned)CAP) {
                    queued = true;
                    q.p0[idx] = (unsigned long long)p0;
                    q.a[idx] = a;
                    int32_t l32 = (int32_t)len;
                    if (len >= T_HUGE) {
                        const unsigned h = atomicAdd(&q.n_huge, 1u) - hstart;
                        if (h < (unsigned)MAX_HUGE) { q.huge[h] = (int32_t)idx; l32 = -l32; }
                    }
                    q.len[idx] = l32;
                }
            }
            if (!queued) {
                for (int64_t p = p0; p < p0 + len; ++p) {
                    if constexpr (HAS_VAL) f(b_col[p], a * b_val[p]);
                    else f(b_col[p], a);
                }
            }
        }
        __syncthreads();
        const unsigned total = q.n - start;
        const unsigned htotal = q.n_huge - hstart;
        const int nq = (int)(total < (unsigned)CAP ? total : (unsigned)CAP);
        const int nh = (int)(htotal < (unsigned)MAX_HUGE ? htotal : (unsigned)MAX_HUGE);
        for (int i = grp; i < nq; i += NG) {
            const int32_t len = q.len[i];
            if (len > 0 && len < T_LONG) {
                const int64_t p0 = (int64_t)q.p0[i];
                const V a = q.a[i];
                for (int64_t p = p0 + gl; p < p0 + len; p += MED_LANES) {
                    if constexpr (HAS_VAL) f(b_col[p], a * b_val[p]);
                    else f(b_col[p], a);
                }
            }
        }
        for (int i = wave; i < nq; i += NW) {
            const int32_t len = q.len[i];
            if (len >= T_LONG) {
                const int64_t p0 = (int64_t)q.p0[i];
                const V a = q.a[i];
                for (int64_t p = p0 + lane; p < p0 + len; p += WAVE) {
                    if constexpr (HAS_VAL) f(b_col[p], a * b_val[p]);
                    else f(b_col[p], a);
                }
            }
        }
        for (int h = 0; h < nh; ++h) {
            const int i = q.huge[h];
            const int64_t len = -(int64_t)q.len[i];
            const int64_t p0 = (int64_t)q.p0[i];
            const V a = q.a[i];
            for (int64_t p = p0 + tid; p < p0 + len; p += THREADS) {
                if constexpr (HAS_VAL) f(b_col[p], a * b_val[p]);
                else f(b_col[p], a);
            }
        }
        __syncthreads();
        start += total;
        hstart += htotal;
    }
    st.start = start;
    st.hstart = hstart;
}

// Per-wave queue of the wave version.
template <typename V>
struct WaveQueue {
    unsigned long long p0[WAVE];
    int32_t len[WAVE];
    V a[WAVE];
};

// Wave version: the 64 lanes of one wave walk one row; no workgroup barrier.
template <bool HAS_VAL, typename V, typename SegFn, typename F>
__device__ __forceinline__ void wave_traverse(const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
                                              int64_t e0, int64_t e1, SegFn seg, const int32_t *__restrict__ b_col,
                                              const V *__restrict__ b_val, WaveQueue<V> &q, F f)
{
    const int lane = lane_id();
    const int gl = lane & (MED_LANES - 1), grp = lane / MED_LANES;
    for (int64_t base = e0; base < e1; base += WAVE) {
        const int64_t e = base + lane;
        int64_t p0 = 0, len = 0;
        V a = V();
        if (e < e1) {
            const int32_t k = a_col[e];
            if constexpr (HAS_VAL) a = a_val[e];
            seg(k, p0, len);
        }
        const bool queued = len >= T_MED;
        const unsigned long long mask = __ballot(queued);
        if (queued) {
            const int idx = __popcll(mask & ((1ull << lane) - 1ull));
            q.p0[idx] = (unsigned long long)p0;
            q.len[idx] = (int32_t)len;
            q.a[idx] = a;
        } else {
            for (int64_t p = p0; p < p0 + len; ++p) {
                if constexpr (HAS_VAL) f(b_col[p], a * b_val[p]);
                else f(b_col[p], a);
            }
        }
        wave_sync();
        const int nq = __popcll(mask);
        for (int i = grp; i < nq; i += WAVE / MED_LANES) {
            const int32_t l = q.len[i];
            if (l < T_LONG) {
                const int64_t s0 = (int64_t)q.p0[i];
                const V aa = q.a[i];
                for (int64_t p = s0 + gl; p < s0 + l; p += MED_LANES) {
                    if constexpr (HAS_VAL) f(b_col[p], aa * b_val[p]);
                    else f(b_col[p], aa);
                }
            }
        }
        for (int i = 0; i < nq; ++i) {
            const int32_t l = q.len[i];
            if (l >= T_LONG) {
                const int64_t s0 = (int64_t)q.p0[i];
                const V aa = q.a[i];
                for (int64_t p = s0 + lane; p < s0 + l; p += WAVE) {
                    if constexpr (HAS_VAL) f(b_col[p], aa * b_val[p]);
                    else f(b_col[p], aa);
                }
            }
        }
        wave_sync();
    }
}

}  // namespace ocean
