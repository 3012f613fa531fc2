/*
 * Ocean SpGEMM for AMD MI355X (gfx950): C = A*B on CSR matrices held in
 * device memory, computed by the estimation-based workflow of the Ocean paper:
 * an analysis step, a per-row size prediction (HyperLogLog estimate, exact
 * symbolic count, or the product-count upper bound), binned Gustavson
 * accumulation in LDS / global hash tables with an overflow-and-retry path,
 * then per-row sort and compaction to canonical CSR.
 *
 * Plain C ABI.  Unless a parameter says "host", every pointer inside an
 * ocean_csr and every array argument is a DEVICE pointer on the current HIP
 * device.  Functions return OCEAN_OK (0) or an error code; they never throw
 * or abort.  ocean_last_error() returns a description of the last failure on
 * the calling thread.
 */
#ifndef OCEAN_SPGEMM_H
#define OCEAN_SPGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A hipStream_t (0 = the null stream).  Kept opaque so that C callers need no HIP headers. */
typedef void *ocean_stream_t;

enum { OCEAN_F64 = 0, OCEAN_F32 = 1 };

enum {
    OCEAN_OK = 0,
    OCEAN_EINVAL = 1, /* null / inconsistent arguments, A.cols != B.rows, dtype mismatch, invalid CSR content,
                         or a single row of A*B with 2^31 or more intermediate products */
    OCEAN_EALLOC = 2, /* the allocator could not provide memory */
    OCEAN_EHIP = 3    /* a HIP runtime call failed */
};

/* Workflows of Table 1 of the paper.  AUTO applies the table's rule. */
enum { OCEAN_WF_AUTO = 0, OCEAN_WF_UPPER_BOUND = 1, OCEAN_WF_HLL = 2, OCEAN_WF_SYMBOLIC = 3 };

/* How AUTO chooses: Table 1 as printed (thresholds from the options), or the same table with the CR
 * threshold re-derived for MI355X from measured compaction and symbolic rates: it slides from
 * tuned_cr_light (all products in rows that fit the LDS key tables) to tuned_cr_heavy (all in rows that
 * outgrow them); problems with fewer than tuned_min_products products run the two-pass workflow without
 * sketching or sampling (no sampled CR in the statistics then).  Where that
 * rule picks the estimation workflow although the sampled CR is below tuned_cr_bound, the upper-bound
 * workflow runs instead: an estimate with 13 - 18 % error and its expansion factor reserves no less than
 * the product bound then does, and the bound costs no estimation pass and cannot overflow (with the default
 * thresholds, tuned_cr_light above tuned_cr_bound, this is never the case: it matters when tuned_cr_light is
 * lowered). */
enum { OCEAN_SEL_TABLE1 = 0, OCEAN_SEL_MI355X = 1 };

/*
 * CSR matrix (Section 2.1): row_ptr has rows+1 ascending 0-based offsets,
 * col_idx / val hold the entries of each row contiguously.  Column ids are
 * 32-bit as in the paper; row offsets are 64-bit because nnz(C) can exceed
 * 2^31.  Inputs may hold unsorted rows, repeated columns and explicit zeros
 * (repeated columns add up).  Outputs are canonical: strictly ascending
 * columns inside each row and one entry per structurally reachable (i, j);
 * numerical cancellation does not remove entries.
 */
typedef struct ocean_csr {
    int64_t rows, cols, nnz;
    int64_t *row_ptr; /* device, rows+1 */
    int32_t *col_idx; /* device, nnz */
    void *val;        /* device, nnz elements of dtype */
    int32_t dtype;    /* OCEAN_F64 or OCEAN_F32 */
    int32_t reserved;
} ocean_csr;

/*
 * Device-memory provider.  alloc returns 0 and a pointer aligned to at least
 * 256 bytes, usable on the stream passed to the library call; release gives
 * it back.  Both are called on the calling host thread only.  With a NULL
 * allocator the library uses hipMalloc / hipFree.
 */
typedef struct ocean_allocator {
    void *ctx;
    int (*alloc)(void *ctx, size_t bytes, void **ptr);
    void (*release)(void *ctx, void *ptr);
} ocean_allocator;

/* Parameters; ocean_default_options fills in the paper's values (Section 4.3, Table 1) and, for what the paper
 * tuned empirically on its own GPU or leaves to the implementation, the values measured on MI355X. */
typedef struct ocean_options {
    int32_t workflow;                /* OCEAN_WF_*; AUTO = Table 1 */
    int32_t hll_registers;           /* 0 = 32 if ER < 48 else 64 (Section 4.3); or 32 / 64 / 128 */
    double upper_bound_avg_products; /* 64: below this average products/row, bin by the product count */
    double er_threshold;             /* 8 */
    double cr_threshold;             /* 8 */
    double expand_coef;              /* 0 = 1.5, or 2.0 with 32 registers (Section 5.3); else the factor itself */
    double exact_load_coef;          /* table slots per exact output entry on the two-pass path (1.5, Section 2.2) */
    double sample_ratio;             /* 0.03 */
    int32_t sample_min, sample_max;  /* 600, 10000 */
    uint32_t sample_seed;
    double estimate_scale;           /* test hook: every estimate is multiplied by this before binning (1.0) */
    int32_t validate_inputs;         /* 1: check column ids and row offsets on the device first */
    int32_t force_hash_kernels;      /* 1: rows beyond the 8192-slot LDS table always use the hybrid (LDS keys, global
                                        values) and global-table hash kernels, as they do when B's rows are unsorted */
    int32_t assisted_symbolic;       /* assisted symbolic binning (Section 4.1): the key tables of the exact symbolic pass
                                        are sized from products / conservative CR instead of the products.  0: off;
                                        1 (default): whenever the analysis sampled rows, i.e. under OCEAN_WF_AUTO;
                                        2: also sample (sketch + 3 % merge) when the workflow is forced to symbolic.
                                        Rows whose table fills up are recounted with product-sized tables */
    double assist_sigmas;            /* conservative CR = max(1, mean - assist_sigmas * std) of the per-row ratio
                                        products / estimate over the sampled rows (1.0) */
    int32_t bitmap_query;            /* dense accumulators read a column's presence bit and set it only when it is
                                        clear (Section 4.1): 0 never; 1 always in the numeric pass; 2 also in the
                                        bitmap kernel of the symbolic pass (where it measured slower); -1 (default)
                                        in the numeric pass when a sampled CR is known and >= bitmap_query_cr */
    int32_t esc_short_rows;          /* 1: rows with at most 16 / 32 intermediate products are accumulated by
                                        expand-sort-compress, 4 / 2 rows per wave, wherever accumulators are sized from
                                        the product bound (upper-bound workflow, retry; Section 3.3); 0 (default): by the
                                        8-lanes-per-row hash kernel, which measured faster on this GPU (one product per
                                        lane leaves the sort network's lanes a quarter as busy) */
    double bitmap_query_cr;          /* 2.0 (Section 4.3) */
    int32_t selector;                /* OCEAN_SEL_MI355X (default) or OCEAN_SEL_TABLE1 (the paper's thresholds as printed) */
    int32_t compact_in_place;        /* estimation workflows: rows are compacted inside the temporary output, which then
                                        becomes C (col_idx / val stay as large as the reservation), instead of into a
                                        second allocation (Section 5.2, memory overhead).  0 never, 1 whenever the rows
                                        allow it, -1 (default) when both copies together would exceed 40 % of the
                                        device's memory or the second allocation fails */
    double tuned_cr_light;           /* 3.0 */
    double tuned_cr_heavy;           /* 4.5 */
    double tuned_min_products;       /* 4194304 */
    double tuned_cr_bound;           /* 1.5; 0 = the estimation workflow is never replaced by the upper bound */
    double bound_load_coef;          /* table slots per intermediate product of the row: what the upper-bound workflow asks
                                        for, and the most any workflow asks for (more slots than products are of no
                                        use).  1.15: with 1.0 a row whose products are all distinct fills its table to
                                        the last slot (64 products in 64 slots measured twice as slow as in 256) */
    double estimate_table_coef;      /* estimation workflow: accumulator slots per estimated entry where that is less
                                        than the expansion factor (which still sizes the reserved output).  1.75: with
                                        32 registers the factor 2.0 sends a quarter of the rows of a 234-entries-per-row
                                        input to tables twice the size they need; 0 = the expansion factor itself */
    int32_t dense_range;             /* accumulator selection of Section 3.3: a row whose column range (first to last
                                        column of the rows of B it references) is at most 4096 columns and needs no
                                        more LDS as values + presence bits than the hash table the row would get
                                        (512 slots or more) is accumulated densely over that range.  0 never; 1
                                        (default) when 2 % or more of the sampled rows are such rows (then the ranges
                                        of all rows are computed, one more pass over A); 2 always compute the ranges */
    double sort_b_ratio;             /* detector for the throughput-bound case of the accumulators that keep values in
                                        global memory (Section 5.4): when B's rows are unsorted and the rows that
                                        outgrow the LDS hash tables hold at least sort_b_ratio * nnz(B) products, a copy
                                        of B with sorted rows is made (rows of B up to 4096 entries) so that they run
                                        through the column-window kernel instead.  8.0; 0 = never */
    const ocean_allocator *allocator; /* host pointer, may be NULL */
} ocean_options;

#define OCEAN_MAX_BINS 12
/* stage indices of ocean_stats.stage_ms */
enum {
    OCEAN_ST_ANALYSIS = 0,  /* input check, products per row, ER */
    OCEAN_ST_SKETCH = 1,    /* one HLL sketch per row of B */
    OCEAN_ST_SAMPLE = 2,    /* merged sketches of the sampled rows, sampled CR */
    OCEAN_ST_PREDICT = 3,   /* HLL merge+estimate of all rows, or the exact symbolic pass */
    OCEAN_ST_BINNING = 4,   /* row classification, scans, output allocation */
    OCEAN_ST_NUMERIC = 5,   /* accumulation + per-row sort, all bins */
    OCEAN_ST_RETRY = 6,     /* overflow rows recomputed with bound-sized accumulators */
    OCEAN_ST_COMPACT = 7,   /* row sizes -> row_ptr, rows moved to contiguous CSR */
    OCEAN_NUM_STAGES = 8
};

typedef struct ocean_stats {
    int64_t products;          /* P: intermediate products */
    int64_t max_row_products;
    int64_t heavy_products;    /* products of the rows whose product count exceeds the largest LDS hash table (4096) */
    int64_t nnz_c;
    double er;                 /* P / nnz(A) */
    double avg_products;       /* P / rows(A) */
    double sampled_cr;         /* 0 when not computed */
    double cr_mean, cr_std;    /* mean and standard deviation of products / estimate over the sampled rows */
    double assist_cr;          /* the conservative CR the symbolic pass was binned with; 0: binned by products */
    int32_t workflow;          /* the one that ran */
    int32_t hll_registers;     /* 0 when no sketch was built */
    int32_t sampled_rows;
    int32_t fell_back;         /* 1: estimation workflow abandoned for the two-pass one (out of memory) */
    int64_t rows_per_bin[OCEAN_MAX_BINS];          /* numeric bins: the hash bins of ocean_bin_layout, then (at index
                                                      n_numeric) the rows of the dense accumulator over the row's range */
    int64_t symbolic_rows_per_bin[OCEAN_MAX_BINS]; /* symbolic bins (two-pass workflow) */
    int64_t overflow_rows;
    int64_t symbolic_overflow_rows; /* rows whose assisted key table filled up and that were recounted */
    int64_t temp_slots;        /* output slots reserved before compaction (estimation workflows) */
    int64_t peak_bytes;        /* largest total obtained from the allocator at one time */
    int32_t compacted_in_place; /* 1: C's col_idx / val are the temporary output, compacted in place */
    int32_t b_sorted_copy;      /* 1: the numeric pass read a copy of B with sorted rows (see sort_b_ratio) */
    int32_t dense_range_rows;   /* sampled rows for which the dense accumulator over the row's column range would be
                                   chosen (with dense_range = 1 and a sample taken) */
    float stage_ms[OCEAN_NUM_STAGES];
    float total_ms;            /* host wall clock of the call */
    /* per numeric bin (first attempt only): kernel time from events on the call's stream, and the
     * work it covered: intermediate products, entries of A read, entries of C produced.  When B's rows
     * are sorted and some row outgrows the largest LDS hash table, the rows of the last three bins of
     * ocean_bin_layout run in ONE launch of the column-window kernel: its time is reported under the last
     * bin and bin_ms of the two before it is 0. */
    float bin_ms[OCEAN_MAX_BINS];
    int64_t bin_products[OCEAN_MAX_BINS];
    int64_t bin_nnz_a[OCEAN_MAX_BINS];
    int64_t bin_nnz_c[OCEAN_MAX_BINS];
} ocean_stats;

void ocean_default_options(ocean_options *opt /* host */);

/*
 * C = A*B (paper, Section 2.1 problem statement; workflow of Figure 4).
 * A is m x k, B is k x n, both borrowed and never modified; dtype(A) ==
 * dtype(B) == dtype(C).  C is a host struct the call fills in: its three
 * arrays come from opt->allocator (or hipMalloc) and belong to the caller,
 * who returns them with ocean_csr_release.  col_idx / val may be larger than
 * nnz entries.  opt and stats are host pointers and may be NULL.  Work is
 * enqueued on `stream`; the call blocks the host wherever a total has to be
 * read back to size an allocation and returns after the stream has drained,
 * so C is complete on return.  On failure *C is zeroed and everything the
 * call obtained from the allocator has been released.  The result is exact
 * whatever the estimates were (Section 3.2, overflow handling).
 */
int ocean_spgemm(const ocean_csr *A, const ocean_csr *B, ocean_csr *C, const ocean_options *opt,
                 ocean_stats *stats, ocean_stream_t stream);

/* Return C's arrays to the allocator that produced them (NULL = hipFree) and zero the struct. */
int ocean_csr_release(ocean_csr *C, const ocean_allocator *allocator);

/*
 * Analysis (Section 3.2): prod[i] = sum over stored A_ik of nnz(B_k), the
 * number of intermediate products and an upper bound of nnz(C_i).  prod:
 * device int64[A->rows].  total / max_row: host outputs, may be NULL.
 * Blocks until done.  Column ids of A outside [0, B->rows), and row offsets of
 * A that are negative, descending or beyond A->nnz, give OCEAN_EINVAL: such
 * offsets are never dereferenced.
 */
int ocean_row_products(const ocean_csr *A, const ocean_csr *B, int64_t *prod, int64_t *total, int64_t *max_row,
                       ocean_stream_t stream);

/*
 * ocean_row_products for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same kernels as ocean_row_products; the per-row scratch they
 * need (4 + 4 bytes per row of A, and the call's device scalars) lives in a
 * fixed array inside the library's code object, 8 MiB + 256 B per GPU, held
 * until the process ends.  Hence A->rows <= OCEAN_NOALLOC_MAX_ROWS; more rows
 * give OCEAN_EINVAL and nothing is launched.  The call allocates and frees
 * nothing, does not synchronise and reads nothing back: it enqueues its
 * kernels on `stream` and returns.  prod: device int64[A->rows].  totals:
 * device int64[3], written by the last kernel: {P, largest prod[i], flags};
 * flags bit 0: a row offset of A was negative, descending or beyond A->nnz
 * (such rows count as empty), bit 2: a column id of A was outside
 * [0, B->rows) (such entries are skipped).  Every call on one GPU uses that
 * GPU's one array: calls that overlap on the same GPU (two streams, two
 * threads) race and must be serialised by the caller.  ocean_init resolves
 * the array's device address for the current device ahead of time (otherwise
 * the first call on a device does it); call it outside graph capture.
 */
#define OCEAN_NOALLOC_MAX_ROWS (1 << 20)
int ocean_init(void);
int ocean_row_products_noalloc(const ocean_csr *A, const ocean_csr *B, int64_t *prod, int64_t *totals /* device */,
                               ocean_stream_t stream);

/*
 * HLL construct (Sections 2.4, 3.1): one sketch of m one-byte registers per
 * row of B, sketches: device uint8[B->rows * m], m in {32, 64, 128}.
 * Register index = low log2(m) bits of the 32-bit hash, register value =
 * 1 + leading zeros of the remaining bits (0 = empty).  Asynchronous on stream.
 */
int ocean_hll_sketch_rows(const ocean_csr *B, int32_t m, uint8_t *sketches, ocean_stream_t stream);

/*
 * HLL merge + estimate (Section 3.1): for each selected row i of A the
 * element-wise maximum of the sketches of the rows of B it references, and
 * the cardinality estimate of that merged sketch.  rows: device int64[n_rows]
 * row ids, or NULL for rows 0..n_rows-1 (then n_rows must be A->rows).
 * prod / b_cols: when prod is non-NULL (device int64[A->rows]) the estimate
 * is limited to [longest referenced row of B, min(prod[i], b_cols)].
 * est: device double[n_rows].  merged: device uint8[n_rows*m] or NULL.
 * b_row_ptr: device, B's row offsets (needed for the lower limit; may be NULL
 * when prod is NULL).  Asynchronous on stream.
 */
int ocean_hll_merge_estimate(const ocean_csr *A, const uint8_t *sketches, int32_t m, const int64_t *rows,
                             int64_t n_rows, const int64_t *prod, const int64_t *b_row_ptr, int64_t b_cols,
                             double *est, uint8_t *merged, ocean_stream_t stream);

/*
 * Exact symbolic pass (Section 2.3): nnz_per_row[i] = number of distinct
 * output columns of row i; device int32[A->rows].  Blocks until done.
 */
int ocean_symbolic(const ocean_csr *A, const ocean_csr *B, int32_t *nnz_per_row, const ocean_options *opt,
                   ocean_stats *stats, ocean_stream_t stream);

/* Host-only helpers of the analysis step (Section 4.3, Table 1). */
int32_t ocean_select_workflow(double avg_products, double er, double cr, const ocean_options *opt);
/* The choice under OCEAN_SEL_MI355X (see above); products / heavy_products as in ocean_stats. */
int32_t ocean_select_workflow_tuned(double avg_products, double er, double cr, double products, double heavy_products,
                                    const ocean_options *opt);
int32_t ocean_hll_register_count(double er, const ocean_options *opt);
int64_t ocean_sample_size(int64_t rows, const ocean_options *opt);
/* rows_out: host int64[ocean_sample_size(rows)], ascending row ids of the stratified sample. */
int ocean_sample_rows(int64_t rows, const ocean_options *opt, int64_t *rows_out);

/* Number of numeric / symbolic bins and the table slots of each (host arrays of OCEAN_MAX_BINS). */
int ocean_bin_layout(int32_t *numeric_slots, int32_t *n_numeric, int32_t *symbolic_slots, int32_t *n_symbolic);

/*
 * The calls that read totals back keep, per host thread, a small pinned host buffer and the events behind
 * ocean_stats' timings from one call to the next.  ocean_finalize releases those of the calling thread (they
 * are created again on the next call); call it before the thread ends or the library is unloaded.
 */
int ocean_finalize(void);

const char *ocean_last_error(void);
int ocean_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OCEAN_SPGEMM_H */
