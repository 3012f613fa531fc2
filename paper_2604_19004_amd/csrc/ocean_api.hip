// C-ABI entry points and host orchestration of the Ocean SpGEMM pipeline
// (workflow of the paper's Figure 4: analysis -> size prediction -> binning ->
// numeric accumulation -> overflow retry -> sort/compaction).
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "ocean_internal.hpp"

using namespace ocean;

namespace {

thread_local std::string g_err;

int fail(int code, const std::string &msg)
{
    g_err = msg;
    return code;
}

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e__ = (expr);                                                                        \
        if (e__ != hipSuccess)                                                                          \
            return fail(OCEAN_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__));                \
    } while (0)

#define OC_TRY(expr)                   \
    do {                               \
        int rc__ = (expr);             \
        if (rc__ != OCEAN_OK) return rc__; \
    } while (0)

// Device scalars of one call; zeroed at the start.
struct Scalars {
    unsigned long long totals[4];                 // [0]: a total copied here to be read back (slots reserved, nnz(C))
    unsigned long long bin_count[OCEAN_MAX_BINS];
    unsigned long long bin_cursor[OCEAN_MAX_BINS];
    unsigned long long bin_prod[OCEAN_MAX_BINS];  // intermediate products of the rows of each bin
    unsigned long long max_cap;
    unsigned long long ovf_count;
    unsigned long long queue[4];
    double sample_sums[6];                        // products, estimates, per-row CR, its squares, rows counted
    int32_t flags;
    int32_t pad;
    unsigned long long bin_work[3 * OCEAN_MAX_BINS];   // products, entries of A, entries of C per numeric bin
    unsigned long long near_pairs[2];             // sampled entries of B, and those whose successor's column is 1 .. 4 larger
    unsigned long long row_totals[ROW_TOTAL_SLOTS * ROW_TOTAL_STRIDE];   // totals of the row-products pass, by slot
};

// P, largest row, products of the heavy rows from the slots of a fetched Scalars
void sum_row_totals(const Scalars *h, unsigned long long (&out)[3])
{
    out[0] = out[1] = out[2] = 0;
    for (int i = 0; i < ROW_TOTAL_SLOTS; ++i) {
        const unsigned long long *slot = h->row_totals + (size_t)i * ROW_TOTAL_STRIDE;
        out[0] += slot[0];
        out[1] = slot[1] > out[1] ? slot[1] : out[1];
        out[2] += slot[2];
    }
}

constexpr size_t ALIGN = 256;
inline size_t up(size_t b) { return (b + ALIGN - 1) / ALIGN * ALIGN; }

struct Ctx {
    hipStream_t s = nullptr;
    const ocean_allocator *al = nullptr;
    std::vector<std::pair<void *, size_t>> live;
    size_t cur = 0, peak = 0;
    int n_cu = 256;
    int lanes_div = 1;      // see lanes_div_of
    Scalars *h = nullptr;   // pinned host mirror
    // stage timing
    std::vector<hipEvent_t> ev;
    std::vector<int> ev_stage;
    std::vector<std::pair<int, int>> bin_ev;   // (numeric bin, index of the event recorded before its launch)
    // column-window boundary table of B for the dense kernel (null: heavy rows use global hash tables)
    uint32_t *bw = nullptr;
    int n_win = 0;
    bool query_bitmap = false;
    bool fine_buckets = false;

    void *alloc(size_t bytes)
    {
        if (bytes == 0) bytes = ALIGN;
        void *p = nullptr;
        if (al && al->alloc) {
            if (al->alloc(al->ctx, bytes, &p) != 0) p = nullptr;
        } else {
            if (hipMalloc(&p, bytes) != hipSuccess) { (void)hipGetLastError(); p = nullptr; }
        }
        if (p) {
            live.emplace_back(p, bytes);
            cur += bytes;
            peak = cur > peak ? cur : peak;
        }
        return p;
    }
    void release(void *p)
    {
        if (!p) return;
        for (size_t i = 0; i < live.size(); ++i)
            if (live[i].first == p) {
                cur -= live[i].second;
                live.erase(live.begin() + i);
                break;
            }
        if (al && al->release) al->release(al->ctx, p);
        else (void)hipFree(p);
    }
    // hand ownership to the caller
    void detach(void *p)
    {
        for (size_t i = 0; i < live.size(); ++i)
            if (live[i].first == p) { live.erase(live.begin() + i); return; }
    }
    void release_all()
    {
        while (!live.empty()) release(live.back().first);
    }
};

struct PinnedHost {
    Scalars *p = nullptr;
    std::vector<hipEvent_t> events;
};
thread_local PinnedHost g_pinned;

// Compute units and memory of the current device, asked for once per device and host thread.
struct DeviceFacts {
    int cus = 0;
    size_t total_mem = 0;
};
const DeviceFacts &device_facts()
{
    static thread_local DeviceFacts cached[64];
    static thread_local DeviceFacts fallback;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        fallback.cus = 256;
        fallback.total_mem = 0;
        return fallback;
    }
    DeviceFacts &f = cached[dev];
    if (f.cus == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) == hipSuccess) {
            f.cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
            f.total_mem = prop.totalGlobalMem;
        } else {
            (void)hipGetLastError();
            f.cus = 256;
        }
    }
    return f;
}

int ctx_init(Ctx &c, const ocean_options *opt, ocean_stream_t stream)
{
    c.s = static_cast<hipStream_t>(stream);
    c.al = opt ? opt->allocator : nullptr;
    c.n_cu = device_facts().cus;
    if (!g_pinned.p) {
        void *p = nullptr;
        HIP_TRY(hipHostMalloc(&p, sizeof(Scalars) + 4096, hipHostMallocPortable));
        g_pinned.p = static_cast<Scalars *>(p);
    }
    c.h = g_pinned.p;
    return OCEAN_OK;
}

int mark(Ctx &c, int stage)
{
    const size_t i = c.ev.size();
    if (g_pinned.events.size() <= i) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        g_pinned.events.push_back(e);
    }
    HIP_TRY(hipEventRecord(g_pinned.events[i], c.s));
    c.ev.push_back(g_pinned.events[i]);
    c.ev_stage.push_back(stage);
    return OCEAN_OK;
}

void collect_times(Ctx &c, ocean_stats *st)
{
    if (!st) return;
    for (int i = 0; i < OCEAN_NUM_STAGES; ++i) st->stage_ms[i] = 0.f;
    for (size_t i = 0; i + 1 < c.ev.size(); ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c.ev[i], c.ev[i + 1]) == hipSuccess && c.ev_stage[i] >= 0) st->stage_ms[c.ev_stage[i]] += ms;
    }
    for (int b = 0; b < OCEAN_MAX_BINS; ++b) st->bin_ms[b] = 0.f;
    for (const auto &be : c.bin_ev) {
        float ms = 0.f;
        if ((size_t)be.second + 1 < c.ev.size() && hipEventElapsedTime(&ms, c.ev[be.second], c.ev[be.second + 1]) == hipSuccess)
            st->bin_ms[be.first] += ms;
    }
}

int fetch_scalars(Ctx &c, const Scalars *dev)
{
    HIP_TRY(hipMemcpyAsync(c.h, dev, sizeof(Scalars), hipMemcpyDeviceToHost, c.s));
    HIP_TRY(hipStreamSynchronize(c.s));
    return OCEAN_OK;
}

Csr view(const ocean_csr *M) { return Csr{M->row_ptr, M->col_idx, M->val, M->rows, M->cols, M->nnz}; }

int check_csr(const ocean_csr *M, const char *name)
{
    if (!M) return fail(OCEAN_EINVAL, std::string(name) + " is null");
    if (M->rows < 0 || M->cols < 0 || M->nnz < 0) return fail(OCEAN_EINVAL, std::string(name) + ": negative size");
    if (M->cols > 0x7fffffffLL || M->rows > 0x7fffffffLL) return fail(OCEAN_EINVAL, std::string(name) + ": more than 2^31-1 rows or columns");
    if (!M->row_ptr) return fail(OCEAN_EINVAL, std::string(name) + ": row_ptr is null");
    if (M->nnz > 0 && (!M->col_idx)) return fail(OCEAN_EINVAL, std::string(name) + ": col_idx is null");
    if (M->dtype != OCEAN_F64 && M->dtype != OCEAN_F32) return fail(OCEAN_EINVAL, std::string(name) + ": unknown dtype");
    return OCEAN_OK;
}

int ilog2_ceil_d(double x, int lo, int hi)
{
    int l = lo;
    while (l < hi && (double)(1ll << l) < x) ++l;
    return l;
}

uint32_t fmix32_host(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85EBCA6Bu;
    h ^= h >> 13;
    h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}

// Per-row work arrays, carved out of one allocation.
struct Work {
    void *base = nullptr;
    Scalars *sc = nullptr;
    bool bins_clean = false;   // the bin counters are still zero from the clearing of all scalars
    int64_t *prod = nullptr;
    int32_t *maxb = nullptr;
    int32_t *cmin = nullptr, *cmax = nullptr;            // column range a row can reach (k_row_spans)
    int32_t *s_cmin = nullptr, *s_cmax = nullptr;        // the same of the sampled rows
    bool spans = false;                                   // cmin / cmax hold the ranges of all rows
    uint8_t *bin = nullptr;
    int32_t *cap = nullptr;
    int32_t *row_nnz = nullptr;
    int32_t *row_nnz2 = nullptr;
    int32_t *nnz_final = nullptr;   // also the exact counts of the symbolic pass
    int32_t *bin_rows = nullptr;
    int64_t *tmp_ptr = nullptr;
    int64_t *tmp_ptr2 = nullptr;
    int64_t *scan_tmp = nullptr;
    double *est = nullptr;
    int64_t *sample_rows = nullptr;
    double *sample_est = nullptr;
};

int work_alloc(Ctx &c, Work &w, int64_t m, int64_t n_sample)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += up(bytes); return o; };
    const size_t mm = (size_t)(m > 0 ? m : 1);
    const size_t o_sc = take(sizeof(Scalars));
    const size_t o_prod = take(mm * 8), o_maxb = take(mm * 4), o_bin = take(mm), o_cap = take(mm * 4);
    const size_t o_nnz = take(mm * 4), o_nnz2 = take(mm * 4), o_nnzf = take(mm * 4), o_rows = take(mm * 4);
    const size_t o_tp = take((mm + 1) * 8), o_tp2 = take((mm + 1) * 8);
    const size_t o_scan = take((size_t)scan_tmp_elems(m) * 8 + 8);
    const size_t o_est = take(mm * 8);
    const size_t o_sr = take((size_t)(n_sample + 1) * 8), o_se = take((size_t)(n_sample + 1) * 8);
    const size_t o_cmin = take(mm * 4), o_cmax = take(mm * 4);
    const size_t o_scmin = take((size_t)(n_sample + 1) * 4), o_scmax = take((size_t)(n_sample + 1) * 4);
    char *b = static_cast<char *>(c.alloc(off));
    if (!b) return fail(OCEAN_EALLOC, "workspace allocation failed");
    w.base = b;
    w.sc = reinterpret_cast<Scalars *>(b + o_sc);
    w.prod = reinterpret_cast<int64_t *>(b + o_prod);
    w.maxb = reinterpret_cast<int32_t *>(b + o_maxb);
    w.bin = reinterpret_cast<uint8_t *>(b + o_bin);
    w.cap = reinterpret_cast<int32_t *>(b + o_cap);
    w.row_nnz = reinterpret_cast<int32_t *>(b + o_nnz);
    w.row_nnz2 = reinterpret_cast<int32_t *>(b + o_nnz2);
    w.nnz_final = reinterpret_cast<int32_t *>(b + o_nnzf);
    w.bin_rows = reinterpret_cast<int32_t *>(b + o_rows);
    w.tmp_ptr = reinterpret_cast<int64_t *>(b + o_tp);
    w.tmp_ptr2 = reinterpret_cast<int64_t *>(b + o_tp2);
    w.scan_tmp = reinterpret_cast<int64_t *>(b + o_scan);
    w.est = reinterpret_cast<double *>(b + o_est);
    w.sample_rows = reinterpret_cast<int64_t *>(b + o_sr);
    w.sample_est = reinterpret_cast<double *>(b + o_se);
    w.cmin = reinterpret_cast<int32_t *>(b + o_cmin);
    w.cmax = reinterpret_cast<int32_t *>(b + o_cmax);
    w.s_cmin = reinterpret_cast<int32_t *>(b + o_scmin);
    w.s_cmax = reinterpret_cast<int32_t *>(b + o_scmax);
    HIP_TRY(hipMemsetAsync(w.sc, 0, sizeof(Scalars), c.s));
    w.bins_clean = true;
    return OCEAN_OK;
}

int zero_bins(Ctx &c, Work &w)
{
    if (w.bins_clean) {   // (the analysis step in between touches none of them but the last row counter, which only
        w.bins_clean = false;   // the retry uses, after a clearing of its own)
        return OCEAN_OK;
    }
    HIP_TRY(hipMemsetAsync(w.sc->bin_count, 0,
                           sizeof(unsigned long long) * (3 * OCEAN_MAX_BINS + 2 + 4), c.s));   // counts, cursors, products, max_cap, ovf, queues
    return OCEAN_OK;
}

// ---- analysis: validation + products per row ------------------------------------------------------
int run_analysis(Ctx &c, Work &w, const Csr &A, const Csr &B, bool validate, ocean_stats *st)
{
    if (validate) HIP_TRY(launch_validate(A, B, &w.sc->flags, w.sc->near_pairs, c.s));
    // (the row list of the bins and the last row counter are free at this point: scratch of the long-row list)
    HIP_TRY(launch_row_products(A, B.rp, B.rows, w.prod, w.maxb, w.sc->row_totals, &w.sc->flags, w.bin_rows,
                                &w.sc->queue[3], c.s));
    OC_TRY(fetch_scalars(c, w.sc));
    unsigned long long tot[3];
    sum_row_totals(c.h, tot);
    if (c.h->flags & 1) return fail(OCEAN_EINVAL, "A is not a valid CSR matrix (row offsets or column ids out of range)");
    if (c.h->flags & 2) return fail(OCEAN_EINVAL, "B is not a valid CSR matrix (row offsets or column ids out of range)");
    if (c.h->flags & 4) return fail(OCEAN_EINVAL, "a column id of A is outside [0, rows(B))");
    if (tot[1] >= (1ull << 31))   // the kernels number the products of a row in 32 bits
        return fail(OCEAN_EINVAL, "a row of A*B has 2^31 or more intermediate products");
    // clustered columns (a quarter or more of B's entries sit within 4 columns of their successor): the hash kernels
    // then order their rows through narrower column buckets (known only when the inputs were checked)
    c.fine_buckets = validate && c.h->near_pairs[0] > 0 && (double)c.h->near_pairs[1] * 4.0 >= (double)c.h->near_pairs[0];
    if (st) {
        st->products = (int64_t)tot[0];
        st->max_row_products = (int64_t)tot[1];
        st->heavy_products = (int64_t)tot[2];
        st->er = A.nnz > 0 ? (double)st->products / (double)A.nnz : 0.0;
        st->avg_products = A.rows > 0 ? (double)st->products / (double)A.rows : 0.0;
    }
    return OCEAN_OK;
}

void sample_rows_of(int64_t rows, const ocean_options &o, int64_t *out);

// ---- exact symbolic pass ---------------------------------------------------------------------------
// assist_cr > 1: assisted binning (Section 4.1) - key tables are sized from products / assist_cr, rows
// whose table fills up report -1 and are recounted in a second round with tables sized from the products.
int run_symbolic(Ctx &c, Work &w, const Csr &A, const Csr &B, int gb_log2, double assist_cr, bool query_bitmap,
                 int32_t *nnz_out, ocean_stats *st)
{
    HIP_TRY(launch_fill_i32(nnz_out, A.rows, 0, c.s));
    // With at most 2^20 columns the bitmap kernel covers a row in one window, and one pass over such a
    // window costs less than building a key table of 16384 or 32768 slots: those two bins go with it
    // (the row lists of consecutive bins are adjacent).
    const bool wide_bitmap = B.cols <= (1 << 20);
    for (int round = 0; round < 2; ++round) {
        const bool assisted = round == 0 && assist_cr > 1.0;
        BinParams bp{};
        bp.mode = 3;
        bp.coef = assisted ? assist_cr : 1.0;
        bp.n_bins = SB_COUNT;
        for (int b = 0; b < SB_COUNT; ++b) bp.slots[b] = kSymbolicSlots[b];
        bp.n_cols = B.cols;
        OC_TRY(zero_bins(c, w));
        HIP_TRY(launch_classify(A.rows, bp, 1.0, w.prod, nullptr, nullptr, round == 0 ? nullptr : nnz_out, w.maxb, w.bin,
                                nullptr, w.sc->bin_count, nullptr, nullptr, c.s));
        HIP_TRY(launch_scatter(A.rows, SB_COUNT, w.bin, w.sc->bin_count, w.sc->bin_cursor, w.bin_rows, c.s));
        OC_TRY(fetch_scalars(c, w.sc));
        int64_t start[SB_COUNT + 1];
        start[0] = 0;
        for (int b = 0; b < SB_COUNT; ++b) {
            start[b + 1] = start[b] + (int64_t)c.h->bin_count[b];
            if (st && round == 0) st->symbolic_rows_per_bin[b] = (int64_t)c.h->bin_count[b];
        }
        for (int b = SB_COUNT - 1; b >= 0; --b) {
            SymLaunch l{w.bin_rows + start[b], start[b + 1] - start[b], b, query_bitmap, assisted};
            if (wide_bitmap && (b == SB_S16K || b == SB_S32K)) continue;
            if (wide_bitmap && b == SB_BITMAP) {
                l.rows = w.bin_rows + start[SB_S16K];
                l.count = start[SB_COUNT] - start[SB_S16K];
            }
            if (l.count == 0) continue;
            const int n_wg = (int)(l.count < c.n_cu ? l.count : c.n_cu);
            HIP_TRY(launch_symbolic_bin(A, B, l, gb_log2, nnz_out, n_wg, &w.sc->queue[round], c.s));
        }
        if (!assisted) break;
        HIP_TRY(launch_count_overflow(A.rows, nnz_out, &w.sc->ovf_count, c.s));
        OC_TRY(fetch_scalars(c, w.sc));
        if (st) st->symbolic_overflow_rows = (int64_t)c.h->ovf_count;
        if (c.h->ovf_count == 0) break;
    }
    return OCEAN_OK;
}

// ---- sampled compression ratio (Section 3.2) and its spread over the sample (Section 4.1) ------------
// With B given (dense_range = 1) the column ranges of the sampled rows are looked at too: S->dense_range_rows is
// the number of sampled rows for which the dense accumulator over the row's range would be chosen.
int run_sample(Ctx &c, Work &w, const Csr &A, const Csr *B, int vbytes, int64_t n_cols, const uint8_t *sketches, int m_regs,
               int64_t n_sample, const ocean_options &o, ocean_stats *S)
{
    HIP_TRY(launch_sample_rows(A.rows, n_sample, o.sample_seed, w.sample_rows, c.s));   // (= sample_rows_of on the host)
    HIP_TRY(launch_hll_merge(A, sketches, m_regs, w.sample_rows, n_sample, w.prod, w.maxb, nullptr, n_cols, w.sample_est,
                             nullptr, c.lanes_div, c.s));
    const bool ranges = B != nullptr && o.dense_range == 1;
    if (ranges) HIP_TRY(launch_row_spans(A, *B, w.sample_rows, n_sample, w.s_cmin, w.s_cmax, c.s));
    HIP_TRY(launch_sample_reduce(w.sample_rows, n_sample, w.prod, w.sample_est, ranges ? w.s_cmin : nullptr, w.s_cmax, n_cols,
                                 vbytes, o.bound_load_coef, w.sc->sample_sums, c.s));
    OC_TRY(fetch_scalars(c, w.sc));
    const double *ss = c.h->sample_sums;
    S->dense_range_rows = (int32_t)ss[5];
    S->sampled_cr = ss[1] > 0.0 ? ss[0] / ss[1] : 1.0;
    S->sampled_rows = (int32_t)n_sample;
    if (ss[4] > 0.0) {
        S->cr_mean = ss[2] / ss[4];
        const double var = ss[3] / ss[4] - S->cr_mean * S->cr_mean;
        S->cr_std = var > 0.0 ? std::sqrt(var) : 0.0;
    }
    return OCEAN_OK;
}

// The compression ratio the symbolic pass may count on (Section 4.1: "conservative estimate" from the mean
// and standard deviation over the sample): assist_sigmas standard deviations below the mean, at least 1.
double conservative_cr(const ocean_stats *S, const ocean_options &o)
{
    if (S->sampled_rows <= 0 || !(S->cr_mean > 0.0)) return 1.0;
    const double v = S->cr_mean - o.assist_sigmas * S->cr_std;
    return v > 1.0 ? v : 1.0;
}

// ---- numeric bins ------------------------------------------------------------------------------------
// Launches every non-empty bin, largest tables first.  Scratch for the hybrid
// and global bins is obtained here and kept until the caller releases all.
int run_numeric(Ctx &c, Work &w, const Csr &A, const Csr &B, int dtype, int gb_log2, const unsigned long long *count,
                const unsigned long long * /*bin_prod*/, int64_t max_cap_global, double global_coef, const int64_t *out_ptr, int32_t *out_col, void *out_val,
                int32_t *row_nnz, int queue_base, int stage, bool time_bins, bool esc)
{
    // With the window table, the column-window kernel takes every row beyond the 4096-slot table (measured:
    // a row of the 8192-slot bin costs less there than a hash table of its own; smaller rows do not).
    constexpr int HEAVY_FROM = NB_S8K;
    int64_t start[NB_ALL + 1];
    start[0] = 0;
    for (int b = 0; b < NB_ALL; ++b) start[b + 1] = start[b] + (int64_t)count[b];
    const size_t vbytes = dtype == OCEAN_F64 ? 8 : 4;
    for (int b = NB_ALL - 1; b >= 0; --b) {
        NumLaunch l{};
        l.rows = w.bin_rows + start[b];
        l.count = start[b + 1] - start[b];
        l.bin = b;
        l.out_ptr = out_ptr;
        l.out_col = out_col;
        l.out_val = out_val;
        l.row_nnz = row_nnz;
        l.coef = global_coef;
        l.fine_buckets = c.fine_buckets;
        if (b == NB_DSPAN) {   // rows whose column range got them the dense accumulator over that range
            l.cmin = w.cmin;
            l.query_bitmap = c.query_bitmap;
        }
        if (c.bw != nullptr && b >= HEAVY_FROM && b < NB_GLOBAL) continue;   // went with the last bin, see below
        if (!esc && b == NB_E16) continue;   // same kernel as the 32-slot bin: one launch for both (adjacent row lists)
        if (!esc && b == NB_G8) {
            l.rows = w.bin_rows + start[NB_E16];
            l.count = start[NB_G8 + 1] - start[NB_E16];
        }
        if (c.bw != nullptr && b == NB_GLOBAL) {
            // the windowed kernel takes the rows of those bins in one launch (their row lists are adjacent)
            l.rows = w.bin_rows + start[HEAVY_FROM];
            l.count = start[NB_GLOBAL + 1] - start[HEAVY_FROM];
            // longest rows first (the kernel takes rows from the end of the list); skipped when memory is short
            const size_t sort_bytes = sort_rows_scratch_bytes(l.count);
            void *sort_tmp = sort_bytes ? c.alloc(sort_bytes) : nullptr;
            if (sort_tmp)
                HIP_TRY(launch_sort_rows_by_products(w.prod, w.bin_rows + start[HEAVY_FROM], l.count, sort_tmp, c.s));
        }
        if (l.count == 0) continue;
        if (b == NB_HYBRID) {
            l.n_wg = (int)(l.count < c.n_cu ? l.count : c.n_cu);
            const size_t bytes = (size_t)l.n_wg * 32768 * vbytes;
            l.slab = c.alloc(bytes);
            l.pairs = l.slab ? c.alloc((size_t)l.n_wg * 32768 * 8) : nullptr;
            if (!l.slab || !l.pairs) return fail(OCEAN_EALLOC, "value slab allocation failed");
            HIP_TRY(hipMemsetAsync(l.slab, 0, bytes, c.s));
            l.queue = &w.sc->queue[queue_base];
        } else if (b == NB_GLOBAL && c.bw != nullptr) {
            l.bw = c.bw;
            l.n_win = c.n_win;
            l.query_bitmap = c.query_bitmap;
            const int64_t resident = (int64_t)c.n_cu * heavy_workgroups_per_cu();
            l.n_wg = (int)(l.count < resident ? l.count : resident);
            l.queue = &w.sc->queue[queue_base + 1];
        } else if (b == NB_GLOBAL) {
            int gbits = 10;
            while (gbits < 31 && (double)(1ll << gbits) < global_coef * (double)max_cap_global) ++gbits;
            int n_wg = (int)(l.count < c.n_cu ? l.count : c.n_cu);
            void *gk = nullptr, *gv = nullptr;
            for (;;) {
                const size_t slots = (size_t)n_wg << gbits;
                gk = c.alloc(slots * 4);
                gv = gk ? c.alloc(slots * vbytes) : nullptr;
                if (gk && gv) break;
                if (gk) c.release(gk);
                gk = nullptr;
                if (n_wg == 1) return fail(OCEAN_EALLOC, "global hash table allocation failed");
                n_wg = n_wg / 2;
            }
            const size_t slots = (size_t)n_wg << gbits;
            HIP_TRY(hipMemsetAsync(gk, 0xFF, slots * 4, c.s));
            HIP_TRY(hipMemsetAsync(gv, 0, slots * vbytes, c.s));
            l.gkeys = static_cast<int32_t *>(gk);
            l.gvals = gv;
            l.gbits = gbits;
            l.n_wg = n_wg;
            l.queue = &w.sc->queue[queue_base + 1];
        }
        if (time_bins) {
            c.bin_ev.emplace_back(b, (int)c.ev.size());
            OC_TRY(mark(c, stage));
        }
        if (esc && (b == NB_E16 || b == NB_G8)) {
            // sizes come from the product bound: a row of these bins has at most 16 / 32 products (Section 3.3, ESC)
            EscLaunch e{l.rows, l.count, b == NB_E16 ? 16 : 32, out_ptr, out_col, out_val, row_nnz};
            HIP_TRY(launch_numeric_esc(A, B, dtype, e, c.s));
            continue;
        }
        HIP_TRY(launch_numeric_bin(A, B, dtype, l, gb_log2, c.s));
    }
    if (time_bins) OC_TRY(mark(c, stage));
    return OCEAN_OK;
}

// ---- compaction inside the temporary output (Section 5.2: "a small auxiliary buffer can compact
// non-consecutive outputs back into the original array") ------------------------------------------------
// Rows lie in the slab in row order, row r from ptr1[r] on, and move down to c_rp[r] <= ptr1[r].  Entries
// are moved in C's order, a range [x, x1) per launch, so that no launch writes where it or a later launch
// still reads: the slab positions not yet consumed start at F(x) (the source of entry x, or for a row that
// comes from the retry's output the start of the next row's region), and F(x) - x, the room gained so far,
// only has to cover the range.  Ranges are copied directly while that room is large (it grows
// geometrically with x when rows were reserved with slack); where it is small the range goes through a
// staging buffer, which only needs the rows after it to stay where they are: that is the condition checked
// first, and it fails only when overflow rows need more room than the rows before them left unused.
// *done = false (nothing moved) when it fails; then the caller needs a separate output.
int compact_in_place(Ctx &c, int64_t m, int dtype, const int64_t *c_rp, const int32_t *nnz1, const int64_t *ptr1,
                     int32_t *t_col, void *t_val, const int64_t *ptr2, const int32_t *r_col, const void *r_val,
                     int64_t nnz_c, bool *done)
{
    constexpr int64_t DIRECT_MIN = 1ll << 20, STAGE = 1ll << 24;
    const size_t vbytes = dtype == OCEAN_F64 ? 8 : 4;
    *done = false;
    std::vector<int64_t> rp((size_t)m + 1), tp((size_t)m + 1);
    std::vector<int32_t> n1((size_t)m);
    HIP_TRY(hipMemcpyAsync(rp.data(), c_rp, (size_t)(m + 1) * 8, hipMemcpyDeviceToHost, c.s));
    HIP_TRY(hipMemcpyAsync(tp.data(), ptr1, (size_t)(m + 1) * 8, hipMemcpyDeviceToHost, c.s));
    HIP_TRY(hipMemcpyAsync(n1.data(), nnz1, (size_t)m * 4, hipMemcpyDeviceToHost, c.s));
    HIP_TRY(hipStreamSynchronize(c.s));
    for (int64_t r = 0; r < m; ++r)
        if (rp[r + 1] > tp[r + 1]) return OCEAN_OK;   // C up to the end of row r would reach into row r+1's region
    int32_t *s_col = nullptr;
    char *s_val = nullptr;
    int64_t x = 0, r = 0;
    while (x < nnz_c) {
        while (rp[r + 1] <= x) ++r;   // row of entry x
        const bool first = n1[r] >= 0;
        if (first && tp[r] == rp[r]) { x = rp[r + 1]; continue; }   // the row already is where it belongs
        const int64_t unread = first ? tp[r] + (x - rp[r]) : tp[r + 1];
        const int64_t room = unread - x;
        if (room >= DIRECT_MIN || x + room >= nnz_c) {
            const int64_t x1 = x + room < nnz_c ? x + room : nnz_c;
            HIP_TRY(launch_compact_range(m, dtype, c_rp, nnz1, ptr1, t_col, t_val, ptr2, r_col, r_val, t_col, t_val, x, x1, 0, c.s));
            x = x1;
        } else {
            if (!s_col) {
                s_col = static_cast<int32_t *>(c.alloc((size_t)STAGE * 4));
                s_val = s_col ? static_cast<char *>(c.alloc((size_t)STAGE * vbytes)) : nullptr;
                if (!s_col || !s_val) return fail(OCEAN_EALLOC, "staging buffer of the in-place compaction could not be allocated");
            }
            const int64_t x1 = x + STAGE < nnz_c ? x + STAGE : nnz_c;
            HIP_TRY(launch_compact_range(m, dtype, c_rp, nnz1, ptr1, t_col, t_val, ptr2, r_col, r_val, s_col, s_val, x, x1, x, c.s));
            HIP_TRY(hipMemcpyAsync(t_col + x, s_col, (size_t)(x1 - x) * 4, hipMemcpyDeviceToDevice, c.s));
            HIP_TRY(hipMemcpyAsync(static_cast<char *>(t_val) + (size_t)x * vbytes, s_val, (size_t)(x1 - x) * vbytes,
                                   hipMemcpyDeviceToDevice, c.s));
            x = x1;
        }
    }
    *done = true;
    return OCEAN_OK;
}

void fill_defaults(ocean_options *o)
{
    std::memset(o, 0, sizeof(*o));
    o->workflow = OCEAN_WF_AUTO;
    o->hll_registers = 0;
    o->upper_bound_avg_products = 64.0;
    o->er_threshold = 8.0;
    o->cr_threshold = 8.0;
    o->expand_coef = 0.0;
    o->exact_load_coef = 1.5;
    o->sample_ratio = 0.03;
    o->sample_min = 600;
    o->sample_max = 10000;
    o->sample_seed = 1;
    o->estimate_scale = 1.0;
    o->validate_inputs = 1;
    o->force_hash_kernels = 0;
    o->assisted_symbolic = 1;
    o->assist_sigmas = 1.0;
    o->bitmap_query = -1;
    o->esc_short_rows = 0;
    o->compact_in_place = -1;
    o->sort_b_ratio = 8.0;
    o->selector = OCEAN_SEL_MI355X;
    o->tuned_cr_light = 3.0;
    o->tuned_cr_heavy = 4.5;
    o->tuned_min_products = 4194304.0;
    o->tuned_cr_bound = 1.5;
    o->bound_load_coef = 1.15;
    o->estimate_table_coef = 1.75;
    o->dense_range = 1;
    o->bitmap_query_cr = 2.0;
    o->allocator = nullptr;
}

int64_t sample_size_of(int64_t rows, const ocean_options &o)
{
    int64_t want = (int64_t)std::ceil(o.sample_ratio * (double)rows);
    if (want > o.sample_max) want = o.sample_max;
    if (want < o.sample_min) want = o.sample_min;
    return want < rows ? want : rows;
}

void sample_rows_of(int64_t rows, const ocean_options &o, int64_t *out)
{
    const int64_t ns = sample_size_of(rows, o);
    for (int64_t t = 0; t < ns; ++t) {
        const int64_t lo = (int64_t)((__int128)t * rows / ns);
        const int64_t hi = (int64_t)((__int128)(t + 1) * rows / ns);
        const uint32_t h = fmix32_host(o.sample_seed + 0x9E3779B9u * (uint32_t)(t + 1));
        out[t] = lo + (int64_t)(h % (uint64_t)(hi - lo));
    }
}

// Lanes per row in the sketch and merge kernels: a quarter of the usual number when no row has more than 16
// times the average number of products (the rows of A and B are then of similar lengths), see launch_hll_sketch.
// Measured: estimation pass of the clustered input 0.239 -> 0.136 ms, of the Laplacian 0.31 -> 0.083 ms; on the
// power-law input the same setting is 40 - 65 % slower, which is what the test keeps away.
int lanes_div_of(const ocean_stats *S)
{
    return (double)S->max_row_products <= 16.0 * S->avg_products ? 4 : 1;
}

int registers_of(double er, const ocean_options &o)
{
    if (o.hll_registers == 32 || o.hll_registers == 64 || o.hll_registers == 128) return o.hll_registers;
    return er < 48.0 ? 32 : 64;
}

int select_of(double avg, double er, double cr, const ocean_options &o)
{
    if (avg < o.upper_bound_avg_products) return OCEAN_WF_UPPER_BOUND;
    if (er >= o.er_threshold && cr >= o.cr_threshold) return OCEAN_WF_HLL;
    return OCEAN_WF_SYMBOLIC;
}

// Table 1 with its CR threshold re-derived for this GPU (selector = OCEAN_SEL_MI355X).  The paper's 8 was
// "chosen empirically to amortize the cost of output compaction" on an A100 (Section 4.3).  Here the
// compaction copy runs at 4.3 - 5.8 TB/s, so what it has to beat is the symbolic pass it replaces:
// estimation wins when products / r_sym > 2 (4 + v) products / (CR * bw), i.e. CR > 2 (4 + v) r_sym / bw.
// Rows that fit the LDS key tables are counted at r_sym = 250 - 460 G products/s (break-even CR 1.2 - 1.5 by
// the rates alone; with the estimate's own pass, its retries and the larger tables it gives the numeric pass
// the two workflows measure the same at CR 3.3 and two passes win by 14 % at CR 1.03: threshold 3),
// rows that outgrow them go through the bitmap kernel at about 1.4 T products/s (break-even CR above 4.5).
// So the threshold slides between the two with the share of the products that heavy rows hold.  Small
// problems (below tuned_min_products) run the two-pass workflow unsampled: there the sketches and the sample
// cost more than any choice between the workflows can gain (4096 rows of 8 entries: 0.29 ms sampled, 0.24 ms not).
int select_tuned(double avg, double er, double cr, double products, double heavy_products, const ocean_options &o)
{
    if (avg < o.upper_bound_avg_products) return OCEAN_WF_UPPER_BOUND;
    if (products < o.tuned_min_products) return OCEAN_WF_SYMBOLIC;
    const double share = products > 0.0 ? heavy_products / products : 0.0;
    const double thr = o.tuned_cr_light + (o.tuned_cr_heavy - o.tuned_cr_light) * share;
    // (an estimate is worth its pass, its expansion factor and its retries only if it undercuts the product
    // bound by more than its own error: below tuned_cr_bound the bound itself is the reservation.  Measured on
    // the rectangular input, CR 1.03: 2.43 ms against 2.61 ms; on the clustered one, CR 3.3: 4.44 against 3.51 ms.
    // With the default thresholds the rule is not reached: below a CR of 3 two passes are faster than either,
    // 2.20 ms on the rectangular input)
    if (er >= o.er_threshold && cr >= thr) return cr < o.tuned_cr_bound ? OCEAN_WF_UPPER_BOUND : OCEAN_WF_HLL;
    return OCEAN_WF_SYMBOLIC;
}

// The whole pipeline.  Everything obtained from the allocator is tracked in c;
// the caller releases what is left on any exit path.
int spgemm_impl(Ctx &c, const ocean_csr *Ain, const ocean_csr *Bin, ocean_csr *C, const ocean_options &o,
                ocean_stats *st)
{
    const Csr A = view(Ain), B = view(Bin);
    const int64_t m = A.rows, n = B.cols;
    const int dtype = Ain->dtype;
    const size_t vbytes = dtype == OCEAN_F64 ? 8 : 4;
    C->rows = m;
    C->cols = n;
    C->dtype = dtype;

    int64_t *c_rp = static_cast<int64_t *>(c.alloc((size_t)(m + 1) * 8));
    if (!c_rp) return fail(OCEAN_EALLOC, "row_ptr allocation failed");
    if (m == 0 || A.nnz == 0 || B.nnz == 0) {
        HIP_TRY(hipMemsetAsync(c_rp, 0, (size_t)(m + 1) * 8, c.s));
        HIP_TRY(hipStreamSynchronize(c.s));
        C->row_ptr = c_rp;
        c.detach(c_rp);
        return OCEAN_OK;
    }

    const int64_t n_sample = sample_size_of(m, o);
    Work w;
    OC_TRY(mark(c, OCEAN_ST_ANALYSIS));
    OC_TRY(work_alloc(c, w, m, n_sample));
    ocean_stats local{};
    ocean_stats *S = st ? st : &local;
    OC_TRY(run_analysis(c, w, A, B, o.validate_inputs != 0, S));
    const int64_t P = S->products;
    if (P == 0) {
        HIP_TRY(hipMemsetAsync(c_rp, 0, (size_t)(m + 1) * 8, c.s));
        HIP_TRY(hipStreamSynchronize(c.s));
        C->row_ptr = c_rp;
        c.detach(c_rp);
        return OCEAN_OK;
    }
    const int gb_log2 = ilog2_ceil_d(S->er, 0, 6);   // lanes sharing one row of B ~ its typical length
    c.lanes_div = lanes_div_of(S);
    const int64_t max_ub = S->max_row_products < n ? S->max_row_products : n;

    // Rows that may outgrow every LDS hash table are accumulated densely over column windows, which
    // needs the window boundaries inside every (sorted) row of B.  Built only when such rows can exist
    // and the table stays small; otherwise, or when a row of B turns out unsorted, they use global tables.
    uint32_t *bw_try = nullptr;
    if (max_ub > kNumericSlots[NB_S8K] && B.nnz < 0xffffffffLL && !o.force_hash_kernels) {
        const int nw = dense_window_count(n, dtype);
        const size_t bytes = (size_t)B.rows * ((size_t)nw + 1) * 4;
        if (nw <= 512 && bytes <= ((size_t)6 << 30)) {   // the heavy-row kernel plans at most 512 windows per row
            bw_try = static_cast<uint32_t *>(c.alloc(bytes));
            if (bw_try) HIP_TRY(launch_window_table(B, dtype, bw_try, &c.n_win, &w.sc->flags, c.s));
        }
    }

    // ---- workflow choice (Table 1) ----
    int workflow = o.workflow;
    int m_regs = 0;
    uint8_t *sketches = nullptr;
    auto build_sketches = [&]() -> int {
        if (sketches) return OCEAN_OK;
        m_regs = registers_of(S->er, o);
        sketches = static_cast<uint8_t *>(c.alloc((size_t)B.rows * m_regs));
        if (!sketches) return fail(OCEAN_EALLOC, "sketch allocation failed");
        OC_TRY(mark(c, OCEAN_ST_SKETCH));
        HIP_TRY(launch_hll_sketch(B, m_regs, sketches, c.lanes_div, c.s));
        return OCEAN_OK;
    };
    if (workflow == OCEAN_WF_AUTO) {
        if (S->avg_products < o.upper_bound_avg_products) {
            workflow = OCEAN_WF_UPPER_BOUND;
        } else if (o.selector == OCEAN_SEL_MI355X && (double)P < o.tuned_min_products) {
            workflow = OCEAN_WF_SYMBOLIC;   // (no sample taken: see select_tuned)
        } else {
            OC_TRY(build_sketches());
            OC_TRY(mark(c, OCEAN_ST_SAMPLE));
            OC_TRY(run_sample(c, w, A, &B, (int)vbytes, n, sketches, m_regs, n_sample, o, S));
            workflow = o.selector == OCEAN_SEL_MI355X
                           ? select_tuned(S->avg_products, S->er, S->sampled_cr, (double)P, (double)S->heavy_products, o)
                           : select_of(S->avg_products, S->er, S->sampled_cr, o);
        }
    }
    if (workflow == OCEAN_WF_SYMBOLIC && o.assisted_symbolic == 2 && S->sampled_rows == 0) {
        OC_TRY(build_sketches());
        OC_TRY(mark(c, OCEAN_ST_SAMPLE));
        OC_TRY(run_sample(c, w, A, &B, (int)vbytes, n, sketches, m_regs, n_sample, o, S));
    }

    // Section 4.1 / 4.3: dense accumulators query the bitmap before writing when the (sampled) CR is at least 2
    // (measured on R-MAT, sampled CR 2.5: the dense windows of the numeric pass gain 2.8 %, the symbolic bitmap kernel,
    // whose only LDS operation per product is that OR, loses 14 %: it queries only when told to, bitmap_query = 2)
    c.query_bitmap = o.bitmap_query >= 1 || (o.bitmap_query < 0 && S->sampled_rows > 0 && S->sampled_cr >= o.bitmap_query_cr);
    const bool query_bitmap = o.bitmap_query == 2;
    Csr Bnum = B;   // what the numeric kernels read: B, or a copy of it with sorted rows (see below)
    bool tried_sorted_copy = false;
    // Section 3.3, accumulator selection: rows whose column range is no larger than the hash table they would get
    // use the dense accumulator over that range.  The ranges of all rows cost a pass over A; it is taken when the
    // sample found such rows (2 % of it or more) or when told to (dense_range = 2), and not when B's rows are known
    // to be out of column order (first and last entry of a row then say nothing about its range).
    if ((o.dense_range == 2 || (o.dense_range == 1 && S->sampled_rows > 0 && (int64_t)S->dense_range_rows * 50 >= S->sampled_rows)) &&
        !(c.h->flags & 8)) {
        HIP_TRY(launch_row_spans(A, B, nullptr, m, w.cmin, w.cmax, c.s));
        w.spans = true;
    }
    int32_t *t_col = nullptr;   // output region of the first attempt (C itself on the two-pass path)
    void *t_val = nullptr;
    int64_t total_slots = 0;
    const int64_t *out_ptr = nullptr;
    for (;;) {   // at most two rounds: an estimation workflow may fall back to the two-pass one when memory is short
        // ---- size prediction ----
        OC_TRY(mark(c, OCEAN_ST_PREDICT));
        BinParams bp{};
        bp.n_bins = NB_COUNT;
        for (int b = 0; b < NB_COUNT; ++b) bp.slots[b] = kNumericSlots[b];
        bp.n_cols = n;
        if (w.spans) {
            bp.cmin = w.cmin;
            bp.cmax = w.cmax;
            bp.vbytes = (int)vbytes;
        }
        if (workflow == OCEAN_WF_HLL) {
            OC_TRY(build_sketches());
            OC_TRY(mark(c, OCEAN_ST_PREDICT));
            HIP_TRY(launch_hll_merge(A, sketches, m_regs, nullptr, m, w.prod, w.maxb, nullptr, n, w.est, nullptr, c.lanes_div, c.s));
            bp.mode = 1;
            bp.coef = o.expand_coef > 0.0 ? o.expand_coef : (m_regs == 32 ? 2.0 : 1.5);
            bp.table_coef = o.estimate_table_coef;
        } else if (workflow == OCEAN_WF_SYMBOLIC) {
            S->assist_cr = o.assisted_symbolic ? conservative_cr(S, o) : 1.0;
            if (!(S->assist_cr > 1.0)) S->assist_cr = 0.0;
            OC_TRY(run_symbolic(c, w, A, B, gb_log2, S->assist_cr, query_bitmap, w.nnz_final, S));
            bp.mode = 2;
            bp.coef = o.exact_load_coef;
        } else {
            bp.mode = 0;
            bp.coef = 1.0;
        }
        bp.bound_coef = o.bound_load_coef;
        S->workflow = workflow;
        S->hll_registers = m_regs;

        // ---- binning + output placement ----
        OC_TRY(mark(c, OCEAN_ST_BINNING));
        OC_TRY(zero_bins(c, w));
        int64_t *ptr = workflow == OCEAN_WF_SYMBOLIC ? c_rp : w.tmp_ptr;
        HIP_TRY(launch_classify(m, bp, o.estimate_scale, w.prod, w.est, w.nnz_final, nullptr, nullptr, w.bin, w.cap,
                                w.sc->bin_count, w.sc->bin_prod, &w.sc->max_cap, c.s));
        HIP_TRY(launch_scan_i32_to_i64(w.cap, m, ptr, w.scan_tmp, &w.sc->totals[0], c.s));   // totals[0]: total slots
        HIP_TRY(launch_scatter(m, NB_ALL, w.bin, w.sc->bin_count, w.sc->bin_cursor, w.bin_rows, c.s));
        OC_TRY(fetch_scalars(c, w.sc));
        total_slots = (int64_t)c.h->totals[0];
        for (int b = 0; b < NB_ALL; ++b) S->rows_per_bin[b] = (int64_t)c.h->bin_count[b];
        c.bw = (bw_try != nullptr && !(c.h->flags & 8)) ? bw_try : nullptr;
        if (bw_try != nullptr && (c.h->flags & 8) && !tried_sorted_copy && o.sort_b_ratio > 0.0 &&
            (double)S->heavy_products >= o.sort_b_ratio * (double)B.nnz) {
            // Throughput-bound case of the accumulators that keep values in global memory (Section 5.4): B's rows
            // are unsorted, so heavy rows would go to those kernels, and they hold many times more products than B
            // has entries.  Sorting a copy of B once (nnz(B) work) buys them the column-window kernel instead.
            tried_sorted_copy = true;
            int32_t *s_col = static_cast<int32_t *>(c.alloc((size_t)B.nnz * 4));
            void *s_val = s_col ? c.alloc((size_t)B.nnz * vbytes) : nullptr;
            if (s_col && s_val) {
                HIP_TRY(hipMemsetAsync(&w.sc->flags, 0, sizeof(int32_t), c.s));
                HIP_TRY(launch_sort_b_rows(B, dtype, s_col, s_val, &w.sc->flags, c.s));
                Csr Bs = B;
                Bs.col = s_col;
                Bs.val = s_val;
                HIP_TRY(launch_window_table(Bs, dtype, bw_try, &c.n_win, &w.sc->flags, c.s));
                OC_TRY(fetch_scalars(c, w.sc));
                if (!(c.h->flags & (8 | 16))) {
                    Bnum = Bs;
                    c.bw = bw_try;
                    S->b_sorted_copy = 1;
                }
            }
        }
        t_col = static_cast<int32_t *>(c.alloc((size_t)total_slots * 4));
        t_val = t_col ? c.alloc((size_t)total_slots * vbytes) : nullptr;
        if (!t_col || !t_val) {
            if (t_col) c.release(t_col);
            t_col = nullptr;
            if (workflow != OCEAN_WF_SYMBOLIC && o.workflow == OCEAN_WF_AUTO) {
                // Section 5.2: with too little memory for the estimation workflow, take the two-pass one
                workflow = OCEAN_WF_SYMBOLIC;
                S->fell_back = 1;
                continue;
            }
            return fail(OCEAN_EALLOC, "output allocation failed");
        }
        out_ptr = ptr;
        break;
    }
    unsigned long long bin_count[OCEAN_MAX_BINS], bin_prod[OCEAN_MAX_BINS];
    std::memcpy(bin_count, c.h->bin_count, sizeof(bin_count));
    std::memcpy(bin_prod, c.h->bin_prod, sizeof(bin_prod));
    const int64_t max_cap = (int64_t)c.h->max_cap;
    double global_coef = workflow == OCEAN_WF_SYMBOLIC ? o.exact_load_coef : 1.25;

    // ---- numeric ----
    OC_TRY(mark(c, OCEAN_ST_NUMERIC));
    HIP_TRY(launch_fill_i32(w.row_nnz, m, 0, c.s));
    // expand-sort-compress needs every row of its bins to have no more products than lanes (true when the bins come
    // from the product bound and B has at least 32 columns) and column ids that leave room for the lane number
    const bool esc_ok = o.esc_short_rows != 0 && n >= 32 && n <= ESC_MAX_COLS;
    OC_TRY(run_numeric(c, w, A, Bnum, dtype, gb_log2, bin_count, bin_prod, max_cap, global_coef, out_ptr, t_col, t_val, w.row_nnz, 0,
                       OCEAN_ST_NUMERIC, st != nullptr, esc_ok && workflow == OCEAN_WF_UPPER_BOUND));
    if (st) {
        HIP_TRY(hipMemsetAsync(w.sc->bin_work, 0, sizeof(w.sc->bin_work), c.s));
        HIP_TRY(launch_bin_work(m, w.bin, w.prod, A.rp, w.row_nnz, w.sc->bin_work, c.s));
    }

    auto copy_bin_work = [&]() {
        for (int b = 0; b < OCEAN_MAX_BINS; ++b) {
            S->bin_products[b] = (int64_t)c.h->bin_work[b];
            S->bin_nnz_a[b] = (int64_t)c.h->bin_work[OCEAN_MAX_BINS + b];
            S->bin_nnz_c[b] = (int64_t)c.h->bin_work[2 * OCEAN_MAX_BINS + b];
        }
    };
    if (workflow == OCEAN_WF_SYMBOLIC) {
        OC_TRY(mark(c, -1));
        OC_TRY(fetch_scalars(c, w.sc));
        copy_bin_work();
        S->nnz_c = total_slots;
        C->row_ptr = c_rp;
        C->col_idx = t_col;
        C->val = t_val;
        C->nnz = total_slots;
        c.detach(c_rp);
        c.detach(t_col);
        c.detach(t_val);
        return OCEAN_OK;
    }

    // ---- overflow rows: redo them with bound-sized tables (Section 3.2) ----
    S->temp_slots = total_slots;
    OC_TRY(mark(c, workflow == OCEAN_WF_UPPER_BOUND ? OCEAN_ST_COMPACT : OCEAN_ST_RETRY));
    // (sizes from the product bound cannot fall short: nothing to count in the upper-bound workflow, unless rows ran
    // with the dense accumulator over a guessed column range)
    if (workflow != OCEAN_WF_UPPER_BOUND || w.spans) HIP_TRY(launch_count_overflow(m, w.row_nnz, &w.sc->ovf_count, c.s));
    // optimistic: if nothing overflowed this scan already is the final row_ptr
    HIP_TRY(launch_scan_i32_to_i64(w.row_nnz, m, c_rp, w.scan_tmp, &w.sc->totals[0], c.s));
    OC_TRY(fetch_scalars(c, w.sc));
    copy_bin_work();
    const int64_t n_ovf = (int64_t)c.h->ovf_count;
    S->overflow_rows = n_ovf;
    int64_t nnz_c = (int64_t)c.h->totals[0];
    int32_t *r_col = nullptr;
    void *r_val = nullptr;
    if (n_ovf > 0) {
        BinParams bp{};
        bp.mode = 0;
        bp.coef = 1.0;
        bp.bound_coef = o.bound_load_coef;
        bp.n_bins = NB_COUNT;
        for (int b = 0; b < NB_COUNT; ++b) bp.slots[b] = kNumericSlots[b];
        bp.n_cols = n;
        OC_TRY(zero_bins(c, w));
        HIP_TRY(launch_classify(m, bp, 1.0, w.prod, nullptr, nullptr, w.row_nnz, nullptr, w.bin, w.cap, w.sc->bin_count,
                                w.sc->bin_prod, &w.sc->max_cap, c.s));
        HIP_TRY(launch_scan_i32_to_i64(w.cap, m, w.tmp_ptr2, w.scan_tmp, &w.sc->totals[0], c.s));
        HIP_TRY(launch_scatter(m, NB_COUNT, w.bin, w.sc->bin_count, w.sc->bin_cursor, w.bin_rows, c.s));
        OC_TRY(fetch_scalars(c, w.sc));
        const int64_t slots2 = (int64_t)c.h->totals[0];
        r_col = static_cast<int32_t *>(c.alloc((size_t)slots2 * 4));
        r_val = r_col ? c.alloc((size_t)slots2 * vbytes) : nullptr;
        if (!r_col || !r_val) return fail(OCEAN_EALLOC, "retry output allocation failed");
        unsigned long long bc2[OCEAN_MAX_BINS], bp2[OCEAN_MAX_BINS];
        std::memcpy(bc2, c.h->bin_count, sizeof(bc2));
        std::memcpy(bp2, c.h->bin_prod, sizeof(bp2));
        HIP_TRY(launch_fill_i32(w.row_nnz2, m, 0, c.s));
        OC_TRY(run_numeric(c, w, A, Bnum, dtype, gb_log2, bc2, bp2, (int64_t)c.h->max_cap, 1.25, w.tmp_ptr2, r_col, r_val,
                           w.row_nnz2, 2, OCEAN_ST_RETRY, false, esc_ok));
        HIP_TRY(launch_final_nnz(m, w.row_nnz, w.row_nnz2, w.nnz_final, c.s));
        HIP_TRY(launch_scan_i32_to_i64(w.nnz_final, m, c_rp, w.scan_tmp, &w.sc->totals[0], c.s));
        OC_TRY(fetch_scalars(c, w.sc));
        nnz_c = (int64_t)c.h->totals[0];
    }

    // ---- compaction ----
    OC_TRY(mark(c, OCEAN_ST_COMPACT));
    int32_t *c_col = nullptr;
    void *c_val = nullptr;
    bool in_place = false;
    const double both = (double)(total_slots + nnz_c) * (double)(4 + vbytes);
    bool want_in_place = o.compact_in_place == 1;
    if (o.compact_in_place < 0) {
        // two copies of a large output side by side are what makes the estimation workflows run out of memory
        // (Section 5.2): beyond 40 % of the device's memory the rows are compacted inside the slab
        const size_t mem_total = device_facts().total_mem;
        if (mem_total > 0 && both > 0.4 * (double)mem_total) want_in_place = true;
    }
    for (int attempt = 0; attempt < 2 && !c_col; ++attempt) {
        if (want_in_place) {
            OC_TRY(compact_in_place(c, m, dtype, c_rp, w.row_nnz, out_ptr, t_col, t_val, w.tmp_ptr2, r_col, r_val, nnz_c, &in_place));
            if (in_place) { c_col = t_col; c_val = t_val; break; }
        }
        c_col = static_cast<int32_t *>(c.alloc((size_t)nnz_c * 4));
        c_val = c_col ? c.alloc((size_t)nnz_c * vbytes) : nullptr;
        if (c_col && c_val) break;
        if (c_col) c.release(c_col);
        c_col = nullptr;
        if (want_in_place || o.compact_in_place == 0) return fail(OCEAN_EALLOC, "output allocation failed");
        want_in_place = true;   // no room for a second copy: compact inside the slab if the rows allow it
    }
    if (!c_col) return fail(OCEAN_EALLOC, "output allocation failed");
    if (!in_place) {
        const int g_log2 = ilog2_ceil_d((double)nnz_c / (double)m, 2, 6);
        HIP_TRY(launch_compact(m, dtype, c_rp, w.row_nnz, out_ptr, t_col, t_val, w.tmp_ptr2, r_col, r_val, c_col, c_val,
                               g_log2, nnz_c, c.s));
    }
    S->compacted_in_place = in_place ? 1 : 0;
    OC_TRY(mark(c, -1));
    HIP_TRY(hipStreamSynchronize(c.s));
    S->nnz_c = nnz_c;
    C->row_ptr = c_rp;
    C->col_idx = c_col;
    C->val = c_val;
    C->nnz = nnz_c;
    c.detach(c_rp);
    c.detach(c_col);
    c.detach(c_val);
    return OCEAN_OK;
}

// ---- scratch of the entry point that allocates nothing ----------------------------------------------
// Layout: the call's device scalars (one 256-byte aligned block), then the longest referenced row of B per
// row of A, then the list of long rows.  The array lives in every GPU's copy of the code object; the name
// below is only a host-side handle, the device address comes from hipGetSymbolAddress, once per device.
constexpr size_t NOALLOC_SCALARS = (sizeof(Scalars) + ALIGN - 1) / ALIGN * ALIGN;
constexpr size_t NOALLOC_BYTES = NOALLOC_SCALARS + 2 * (size_t)OCEAN_NOALLOC_MAX_ROWS * sizeof(int32_t);
constexpr int NOALLOC_MAX_DEVICES = 64;

}  // namespace

static __device__ __align__(256) unsigned char scratch[NOALLOC_BYTES];

namespace {

std::mutex g_scratch_mu;
unsigned char *g_scratch_ptr[NOALLOC_MAX_DEVICES] = {};

// Device address of `scratch` on the current device (resolved on the first call per device).
int scratch_of_current_device(unsigned char **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return fail(OCEAN_EINVAL, "device ordinal beyond what the library tracks");
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(OCEAN_EHIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
    }
    *out = g_scratch_ptr[dev];
    return OCEAN_OK;
}

}  // namespace

// =====================================================================================================
extern "C" {

void ocean_default_options(ocean_options *opt)
{
    if (opt) fill_defaults(opt);
}

int ocean_spgemm(const ocean_csr *A, const ocean_csr *B, ocean_csr *C, const ocean_options *opt, ocean_stats *stats,
                 ocean_stream_t stream)
{
    g_err.clear();
    if (!C) return fail(OCEAN_EINVAL, "C is null");
    std::memset(C, 0, sizeof(*C));
    if (stats) std::memset(stats, 0, sizeof(*stats));
    OC_TRY(check_csr(A, "A"));
    OC_TRY(check_csr(B, "B"));
    if (A->cols != B->rows) return fail(OCEAN_EINVAL, "A.cols != B.rows");
    if (A->dtype != B->dtype) return fail(OCEAN_EINVAL, "A and B differ in dtype");
    if ((A->nnz > 0 && !A->val) || (B->nnz > 0 && !B->val)) return fail(OCEAN_EINVAL, "val is null");
    ocean_options o;
    if (opt) o = *opt;
    else fill_defaults(&o);
    if (o.workflow < OCEAN_WF_AUTO || o.workflow > OCEAN_WF_SYMBOLIC) return fail(OCEAN_EINVAL, "unknown workflow");
    if (o.selector != OCEAN_SEL_TABLE1 && o.selector != OCEAN_SEL_MI355X) return fail(OCEAN_EINVAL, "unknown selector");
    if (o.hll_registers != 0 && o.hll_registers != 32 && o.hll_registers != 64 && o.hll_registers != 128)
        return fail(OCEAN_EINVAL, "hll_registers must be 0, 32, 64 or 128");
    if (!(o.estimate_scale > 0.0) || !(o.exact_load_coef >= 1.0) || o.expand_coef < 0.0 || !(o.sample_ratio >= 0.0) ||
        o.sample_min < 1 || o.sample_max < o.sample_min)
        return fail(OCEAN_EINVAL, "option out of range");
    const auto t0 = std::chrono::steady_clock::now();
    Ctx c;
    OC_TRY(ctx_init(c, &o, stream));
    int rc = spgemm_impl(c, A, B, C, o, stats);
    if (rc != OCEAN_OK) {
        (void)hipStreamSynchronize(c.s);
        std::memset(C, 0, sizeof(*C));
    } else {
        collect_times(c, stats);
    }
    c.release_all();
    if (stats) {
        stats->peak_bytes = (int64_t)c.peak;
        stats->total_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count();
    }
    return rc;
}

int ocean_csr_release(ocean_csr *C, const ocean_allocator *allocator)
{
    if (!C) return fail(OCEAN_EINVAL, "C is null");
    void *ptrs[3] = {C->row_ptr, C->col_idx, C->val};
    for (void *p : ptrs) {
        if (!p) continue;
        if (allocator && allocator->release) allocator->release(allocator->ctx, p);
        else (void)hipFree(p);
    }
    std::memset(C, 0, sizeof(*C));
    return OCEAN_OK;
}

int ocean_row_products(const ocean_csr *A, const ocean_csr *B, int64_t *prod, int64_t *total, int64_t *max_row,
                       ocean_stream_t stream)
{
    g_err.clear();
    OC_TRY(check_csr(A, "A"));
    OC_TRY(check_csr(B, "B"));
    if (A->cols != B->rows) return fail(OCEAN_EINVAL, "A.cols != B.rows");
    if (!prod && A->rows > 0) return fail(OCEAN_EINVAL, "prod is null");
    Ctx c;
    OC_TRY(ctx_init(c, nullptr, stream));
    const size_t mm = (size_t)(A->rows > 0 ? A->rows : 1);
    char *buf = static_cast<char *>(c.alloc(up(sizeof(Scalars)) + mm * 4));
    if (!buf) return fail(OCEAN_EALLOC, "workspace allocation failed");
    Scalars *sc = reinterpret_cast<Scalars *>(buf);
    int32_t *maxb = reinterpret_cast<int32_t *>(buf + up(sizeof(Scalars)));
    int rc = [&]() -> int {
        HIP_TRY(hipMemsetAsync(sc, 0, sizeof(Scalars), c.s));
        HIP_TRY(launch_row_products(view(A), B->row_ptr, B->rows, prod, maxb, sc->row_totals, &sc->flags, nullptr, nullptr, c.s));
        OC_TRY(fetch_scalars(c, sc));
        unsigned long long tot[3];
        sum_row_totals(c.h, tot);
        if (c.h->flags & 1) return fail(OCEAN_EINVAL, "A is not a valid CSR matrix (row offsets out of range or descending)");
        if (c.h->flags & 4) return fail(OCEAN_EINVAL, "a column id of A is outside [0, rows(B))");
        if (total) *total = (int64_t)tot[0];
        if (max_row) *max_row = (int64_t)tot[1];
        return OCEAN_OK;
    }();
    (void)hipStreamSynchronize(c.s);
    c.release_all();
    return rc;
}

int ocean_finalize(void)
{
    g_err.clear();
    for (hipEvent_t e : g_pinned.events) (void)hipEventDestroy(e);
    g_pinned.events.clear();
    if (g_pinned.p) {
        HIP_TRY(hipHostFree(g_pinned.p));
        g_pinned.p = nullptr;
    }
    return OCEAN_OK;
}

int ocean_init(void)
{
    g_err.clear();
    unsigned char *p = nullptr;
    return scratch_of_current_device(&p);
}

int ocean_row_products_noalloc(const ocean_csr *A, const ocean_csr *B, int64_t *prod, int64_t *totals,
                               ocean_stream_t stream)
{
    g_err.clear();
    OC_TRY(check_csr(A, "A"));
    OC_TRY(check_csr(B, "B"));
    if (A->cols != B->rows) return fail(OCEAN_EINVAL, "A.cols != B.rows");
    if (!totals) return fail(OCEAN_EINVAL, "totals is null");
    if (!prod && A->rows > 0) return fail(OCEAN_EINVAL, "prod is null");
    if (A->rows > OCEAN_NOALLOC_MAX_ROWS)
        return fail(OCEAN_EINVAL, "A has more than OCEAN_NOALLOC_MAX_ROWS rows: the fixed scratch array cannot hold its per-row data");
    unsigned char *base = nullptr;
    OC_TRY(scratch_of_current_device(&base));
    hipStream_t s = static_cast<hipStream_t>(stream);
    Scalars *sc = reinterpret_cast<Scalars *>(base);
    int32_t *maxb = reinterpret_cast<int32_t *>(base + NOALLOC_SCALARS);
    int32_t *long_rows = maxb + OCEAN_NOALLOC_MAX_ROWS;
    // the scalars keep the last call's sums: clear them (a fill kernel, so that the call can be captured
    // into a graph); the per-row arrays are written before they are read
    HIP_TRY(launch_fill_u64(reinterpret_cast<unsigned long long *>(sc), (int64_t)(NOALLOC_SCALARS / 8), 0ull, s));
    HIP_TRY(launch_row_products(view(A), B->row_ptr, B->rows, prod, maxb, sc->row_totals, &sc->flags, long_rows, &sc->queue[3], s));
    HIP_TRY(launch_publish_totals(sc->row_totals, &sc->flags, totals, s));
    return OCEAN_OK;
}

int ocean_hll_sketch_rows(const ocean_csr *B, int32_t m, uint8_t *sketches, ocean_stream_t stream)
{
    g_err.clear();
    OC_TRY(check_csr(B, "B"));
    if (m != 32 && m != 64 && m != 128) return fail(OCEAN_EINVAL, "m must be 32, 64 or 128");
    if (!sketches && B->rows > 0) return fail(OCEAN_EINVAL, "sketches is null");
    HIP_TRY(launch_hll_sketch(view(B), m, sketches, 1, static_cast<hipStream_t>(stream)));
    return OCEAN_OK;
}

int ocean_hll_merge_estimate(const ocean_csr *A, const uint8_t *sketches, int32_t m, const int64_t *rows,
                             int64_t n_rows, const int64_t *prod, const int64_t *b_row_ptr, int64_t b_cols,
                             double *est, uint8_t *merged, ocean_stream_t stream)
{
    g_err.clear();
    OC_TRY(check_csr(A, "A"));
    if (m != 32 && m != 64 && m != 128) return fail(OCEAN_EINVAL, "m must be 32, 64 or 128");
    if (n_rows < 0 || (!rows && n_rows != A->rows)) return fail(OCEAN_EINVAL, "n_rows must equal A.rows when rows is null");
    if (n_rows > 0 && (!sketches || !est)) return fail(OCEAN_EINVAL, "sketches / est is null");
    if (prod && !b_row_ptr) return fail(OCEAN_EINVAL, "b_row_ptr is needed to limit the estimates");
    HIP_TRY(launch_hll_merge(view(A), sketches, m, rows, n_rows, prod, nullptr, prod ? b_row_ptr : nullptr, b_cols, est,
                             merged, 1, static_cast<hipStream_t>(stream)));
    return OCEAN_OK;
}

int ocean_symbolic(const ocean_csr *A, const ocean_csr *B, int32_t *nnz_per_row, const ocean_options *opt,
                   ocean_stats *stats, ocean_stream_t stream)
{
    g_err.clear();
    if (stats) std::memset(stats, 0, sizeof(*stats));
    OC_TRY(check_csr(A, "A"));
    OC_TRY(check_csr(B, "B"));
    if (A->cols != B->rows) return fail(OCEAN_EINVAL, "A.cols != B.rows");
    if (!nnz_per_row && A->rows > 0) return fail(OCEAN_EINVAL, "nnz_per_row is null");
    if (A->rows == 0) return OCEAN_OK;
    ocean_options o;
    if (opt) o = *opt;
    else fill_defaults(&o);
    Ctx c;
    OC_TRY(ctx_init(c, &o, stream));
    ocean_stats local{};
    ocean_stats *S = stats ? stats : &local;
    int rc = [&]() -> int {
        Work w;
        const int64_t n_sample = o.assisted_symbolic == 2 ? sample_size_of(A->rows, o) : 0;
        OC_TRY(work_alloc(c, w, A->rows, n_sample));
        const Csr a = view(A), b = view(B);
        OC_TRY(run_analysis(c, w, a, b, o.validate_inputs != 0, S));
        const int gb_log2 = ilog2_ceil_d(S->er, 0, 6);
        double assist_cr = 0.0;
        if (n_sample > 0 && S->products > 0) {
            const int m_regs = registers_of(S->er, o);
            uint8_t *sketches = static_cast<uint8_t *>(c.alloc((size_t)b.rows * m_regs));
            if (!sketches) return fail(OCEAN_EALLOC, "sketch allocation failed");
            c.lanes_div = lanes_div_of(S);
            HIP_TRY(launch_hll_sketch(b, m_regs, sketches, c.lanes_div, c.s));
            OC_TRY(run_sample(c, w, a, nullptr, 8, b.cols, sketches, m_regs, n_sample, o, S));
            S->hll_registers = m_regs;
            assist_cr = conservative_cr(S, o);
            if (!(assist_cr > 1.0)) assist_cr = 0.0;
        }
        S->assist_cr = assist_cr;
        OC_TRY(run_symbolic(c, w, a, b, gb_log2, assist_cr, o.bitmap_query == 2, nnz_per_row, S));
        HIP_TRY(hipStreamSynchronize(c.s));
        return OCEAN_OK;
    }();
    if (rc != OCEAN_OK) (void)hipStreamSynchronize(c.s);
    c.release_all();
    if (stats) stats->peak_bytes = (int64_t)c.peak;
    return rc;
}

int32_t ocean_select_workflow(double avg_products, double er, double cr, const ocean_options *opt)
{
    ocean_options o;
    if (opt) o = *opt;
    else fill_defaults(&o);
    return select_of(avg_products, er, cr, o);
}

int32_t ocean_select_workflow_tuned(double avg_products, double er, double cr, double products, double heavy_products,
                                    const ocean_options *opt)
{
    ocean_options o;
    if (opt) o = *opt;
    else fill_defaults(&o);
    return select_tuned(avg_products, er, cr, products, heavy_products, o);
}

int32_t ocean_hll_register_count(double er, const ocean_options *opt)
{
    ocean_options o;
    if (opt) o = *opt;
    else fill_defaults(&o);
    return registers_of(er, o);
}

int64_t ocean_sample_size(int64_t rows, const ocean_options *opt)
{
    ocean_options o;
    if (opt) o = *opt;
    else fill_defaults(&o);
    return rows <= 0 ? 0 : sample_size_of(rows, o);
}

int ocean_sample_rows(int64_t rows, const ocean_options *opt, int64_t *rows_out)
{
    ocean_options o;
    if (opt) o = *opt;
    else fill_defaults(&o);
    if (rows <= 0) return OCEAN_OK;
    if (!rows_out) return fail(OCEAN_EINVAL, "rows_out is null");
    sample_rows_of(rows, o, rows_out);
    return OCEAN_OK;
}

int ocean_bin_layout(int32_t *numeric_slots, int32_t *n_numeric, int32_t *symbolic_slots, int32_t *n_symbolic)
{
    if (n_numeric) *n_numeric = NB_COUNT;
    if (n_symbolic) *n_symbolic = SB_COUNT;
    for (int b = 0; b < OCEAN_MAX_BINS; ++b) {
        if (numeric_slots) numeric_slots[b] = b < NB_COUNT ? kNumericSlots[b] : 0;
        if (symbolic_slots) symbolic_slots[b] = b < SB_COUNT ? kSymbolicSlots[b] : 0;
    }
    return OCEAN_OK;
}

const char *ocean_last_error(void) { return g_err.c_str(); }

int ocean_version(void) { return 100; }

}  // extern "C"
