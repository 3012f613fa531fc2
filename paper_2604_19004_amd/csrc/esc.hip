// Expand-sort-compress accumulator for very short rows (paper Section 2.2,
// "ESC"; Section 3.3: chosen only in the upper-bound workflow, by the number of
// intermediate products, several rows at a time; Section 4.3: two configurations).
//
// A row with at most L intermediate products (L = 16 or 32) is handled by L
// lanes of a wave, one product per lane, 64 / L rows per wave and 4 waves per
// workgroup, without a hash table and without a workgroup barrier:
//   expand    the row's entries A_ik are read one per lane, the lengths of their
//             rows of B are prefix-summed inside the group, and lane q fetches
//             product number q (column id, a*b);
//   sort      the column id and the lane number are packed into one 32-bit key
//             (Section 4.2: key and pointer in one word, the pointer bits do not
//             take part in the order because they are the low bits of distinct
//             keys) and sorted by a bitonic network whose exchanges are lane
//             swizzles - no memory; the value follows its key with one lane
//             permute afterwards (indirect sort);
//   compress  equal columns are now neighbours: a suffix sum over runs of equal
//             columns leaves each column's total in its first lane, a ballot
//             numbers those lanes, and they write the row.
#include "ocean_internal.hpp"

namespace ocean {

namespace {

constexpr int32_t ESC_PAD = 0x7fffffff;   // key of a lane without a product: sorts last

// Inclusive prefix sum inside every group of L = 16 or 32 consecutive lanes.
template <int L>
__device__ __forceinline__ uint32_t esc_inclusive_scan(uint32_t v, int sub)
{
    static_assert(L == 16 || L == 32, "half a row pair or a row pair of the wave");
    uint32_t o;
    o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false); v += (sub & 15) >= 1 ? o : 0u;
    o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false); v += (sub & 15) >= 2 ? o : 0u;
    o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false); v += (sub & 15) >= 4 ? o : 0u;
    o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false); v += (sub & 15) >= 8 ? o : 0u;
    if (L == 32) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);   // lane 15 of the row before, into rows 1 and 3
    return v;
}

// Key of the lane `xor_mask` away inside its group of 32 lanes.
template <int XOR>
__device__ __forceinline__ int32_t esc_partner(int32_t key)
{
    return __builtin_amdgcn_ds_swizzle(key, (XOR << 10) | 0x1f);   // bit mode: and 0x1f, or 0, xor XOR
}

template <int K, int J>
__device__ __forceinline__ void esc_compare_exchange(int32_t &key, int sub)
{
    const int32_t other = esc_partner<J>(key);
    const bool ascending = (sub & K) == 0;
    const bool lower = (sub & J) == 0;
    const int32_t lo = key < other ? key : other;
    const int32_t hi = key < other ? other : key;
    key = (lower == ascending) ? lo : hi;
}

// Ascending bitonic sort of one key per lane inside every group of L lanes (keys are distinct or ESC_PAD).
template <int L>
__device__ __forceinline__ void esc_sort(int32_t &key, int sub)
{
    esc_compare_exchange<2, 1>(key, sub);
    esc_compare_exchange<4, 2>(key, sub);
    esc_compare_exchange<4, 1>(key, sub);
    esc_compare_exchange<8, 4>(key, sub);
    esc_compare_exchange<8, 2>(key, sub);
    esc_compare_exchange<8, 1>(key, sub);
    // (the last merge of a group runs ascending in every lane: sub & L == 0)
    esc_compare_exchange<16, 8>(key, sub);
    esc_compare_exchange<16, 4>(key, sub);
    esc_compare_exchange<16, 2>(key, sub);
    esc_compare_exchange<16, 1>(key, sub);
    if (L == 32) {
        esc_compare_exchange<32, 16>(key, sub);
        esc_compare_exchange<32, 8>(key, sub);
        esc_compare_exchange<32, 4>(key, sub);
        esc_compare_exchange<32, 2>(key, sub);
        esc_compare_exchange<32, 1>(key, sub);
    }
}

template <typename V, int L>
struct EscChunk {
    uint32_t excl[L];
    long long pbase[L];
    V a[L];
};

}  // namespace

// rows: the row ids of the bin, every one with at most L intermediate products and column ids below
// 2^(31 - log2 L).  out_ptr / out_col / out_val / row_nnz as in the hash kernels.
template <typename V, int L>
__global__ void __launch_bounds__(256)
k_numeric_esc(const int64_t *__restrict__ a_rp, const int32_t *__restrict__ a_col, const V *__restrict__ a_val,
              const int64_t *__restrict__ b_rp, const int32_t *__restrict__ b_col, const V *__restrict__ b_val,
              const int32_t *__restrict__ rows, int64_t count, const int64_t *__restrict__ out_ptr,
              int32_t *__restrict__ out_col, V *__restrict__ out_val, int32_t *__restrict__ row_nnz)
{
    constexpr int LB = L == 32 ? 5 : 4;
    constexpr int R = 256 / L;   // rows per workgroup
    __shared__ EscChunk<V, L> s_ch[R];
    const int rl = threadIdx.x / L;
    const int sub = threadIdx.x % L;
    const int lane = lane_id();
    const int group_base = lane - sub;
    EscChunk<V, L> &ch = s_ch[rl];

    const int64_t r = (int64_t)blockIdx.x * R + rl;
    const bool live = r < count;
    const int64_t row = live ? rows[r] : 0;
    const int64_t e0 = live ? a_rp[row] : 0;
    const int64_t e1 = live ? a_rp[row + 1] : 0;

    // ---- expand: lane q takes product number q of the row
    int32_t col = -1;
    V val = V();
    uint32_t off = 0;   // products of the entries before this chunk
    const int chunks = (int)wave_max_u32((uint32_t)((e1 - e0 + L - 1) / L));   // the rows of a wave advance together
    for (int c = 0; c < chunks; ++c) {
        const int64_t e = e0 + (int64_t)c * L + sub;
        int64_t p0 = 0;
        uint32_t len = 0;
        V a = V();
        if (e < e1) {
            const int64_t k = a_col[e];
            a = a_val[e];
            p0 = b_rp[k];
            len = (uint32_t)(b_rp[k + 1] - p0);
        }
        const uint32_t incl = esc_inclusive_scan<L>(len, sub);
        const uint32_t total = (uint32_t)__shfl((int)incl, group_base + L - 1, WAVE);
        ch.excl[sub] = incl - len;
        ch.pbase[sub] = (long long)p0 - (long long)(incl - len);
        ch.a[sub] = a;
        wave_sync();
        const uint32_t q = (uint32_t)sub - off;   // this lane's product, counted inside the chunk
        if ((uint32_t)sub >= off && q < total) {
            int pos = 0;
#pragma unroll
            for (int step = L >> 1; step > 0; step >>= 1)
                if (ch.excl[pos + step] <= q) pos += step;   // last entry starting at or before q (skips empty ones)
            const int64_t p = ch.pbase[pos] + (long long)q;
            col = b_col[p];
            val = ch.a[pos] * b_val[p];
        }
        off += total;   // (at most L over the whole row: the bin holds rows with at most L products)
        wave_sync();    // the chunk arrays are rewritten by the next turn
    }

    // ---- sort by column, the lane number in the low bits
    int32_t key = col >= 0 ? (int32_t)(((uint32_t)col << LB) | (uint32_t)sub) : ESC_PAD;
    esc_sort<L>(key, sub);
    const bool valid = key != ESC_PAD;
    const int32_t scol = valid ? (int32_t)((uint32_t)key >> LB) : -1;
    V sval = __shfl(val, group_base + (key & (L - 1)), WAVE);   // (a pad's low bits are all ones: some lane of the group)
    if (!valid) sval = V();

    // ---- compress: total of every run of equal columns, in the run's first lane
#pragma unroll
    for (int d = 1; d < L; d <<= 1) {
        const int32_t ocol = __shfl(scol, lane + d, WAVE);
        const V oval = __shfl(sval, lane + d, WAVE);
        if (sub + d < L && ocol == scol) sval += oval;
    }
    const int32_t pcol = __shfl(scol, lane - 1, WAVE);
    const bool head = valid && (sub == 0 || pcol != scol);
    const unsigned long long heads = __ballot(head);
    const unsigned long long mine = L == 32 ? (heads >> group_base) & 0xffffffffull : (heads >> group_base) & 0xffffull;
    const int n_out = __popcll(mine);
    if (live) {
        const int64_t o = out_ptr[row];
        const int64_t cap = out_ptr[row + 1] - o;
        const bool fits = (int64_t)n_out <= cap && off <= (uint32_t)L;
        if (head && fits) {
            const int at = __popcll(mine & ((1ull << sub) - 1ull));
            out_col[o + at] = scol;
            out_val[o + at] = sval;
        }
        if (sub == 0) row_nnz[row] = fits ? n_out : -1;
    }
}

template <typename V>
static hipError_t esc_dispatch(const Csr &A, const Csr &B, const EscLaunch &l, hipStream_t s)
{
    const V *av = static_cast<const V *>(A.val);
    const V *bv = static_cast<const V *>(B.val);
    V *ov = static_cast<V *>(l.out_val);
    if (l.lanes == 16) {
        const int64_t blocks = (l.count + 15) / 16;
        hipLaunchKernelGGL((k_numeric_esc<V, 16>), dim3((unsigned)blocks), dim3(256), 0, s, A.rp, A.col, av, B.rp, B.col, bv,
                           l.rows, l.count, l.out_ptr, l.out_col, ov, l.row_nnz);
    } else if (l.lanes == 32) {
        const int64_t blocks = (l.count + 7) / 8;
        hipLaunchKernelGGL((k_numeric_esc<V, 32>), dim3((unsigned)blocks), dim3(256), 0, s, A.rp, A.col, av, B.rp, B.col, bv,
                           l.rows, l.count, l.out_ptr, l.out_col, ov, l.row_nnz);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_numeric_esc(const Csr &A, const Csr &B, int dtype, const EscLaunch &l, hipStream_t s)
{
    if (l.count <= 0) return hipSuccess;
    return dtype == OCEAN_F64 ? esc_dispatch<double>(A, B, l, s) : esc_dispatch<float>(A, B, l, s);
}

}  // namespace ocean
