/*
 * sptir.h - C ABI of the hyb(c,k) composable-format SpMM library for gfx950
 * (plus SDDMM on CSR, the other sparse operator of the paper's GNN section).
 *
 * The operations follow the SpMM problem statement of the paper (arXiv
 * 2207.04606): A is sparse in CSR with int32 indices and float32 values, X and
 * Y are dense row-major float32 (the SpMM script of Appendix A), and
 *     Y[i,k] = sum_j A[i,j] * X[j,k]                  (Section 4.2.1).
 * A is first decomposed into the parameterised composable format hyb(c,k) of
 * Section 4.2.1: c column partitions of width w = ceil(n_cols / c); in every
 * partition the row pieces of length l with 2^(i-1) < l <= 2^i form ELL bucket
 * i (i = 0..k), padded to width 2^i.  Row pieces longer than 2^k, on which the
 * paper is silent, are kept unpadded in a CSR remainder per partition.
 *
 * All pointers named "device" are GPU global-memory addresses of the current
 * HIP device; everything else is host memory.  No function throws or aborts;
 * every failure is reported through sptir_status_t and leaves the out
 * parameters untouched.  The library is not re-entrant per hyb object: calls
 * that use the same object must be ordered by the caller.
 */
#ifndef SPTIR_H_
#define SPTIR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPTIR_OK = 0,
  SPTIR_ERR_INVALID_ARG = 1, /* null pointer, negative size, parameter out of range, X/Y alias */
  SPTIR_ERR_UNSORTED = 2,    /* column ids of a row not strictly ascending, or outside [0, n_cols) */
  SPTIR_ERR_OVERFLOW = 3,    /* a count does not fit the index type of its array */
  SPTIR_ERR_ALLOC = 4,       /* the allocator returned NULL */
  SPTIR_ERR_HIP = 5,         /* a HIP runtime call failed; see sptir_last_hip_error() */
  SPTIR_ERR_UNSUPPORTED = 6  /* valid request this build cannot serve (e.g. misaligned X/Y) */
} sptir_status_t;

/*
 * CSR input (axes I = dense_fixed(m), J = sparse_variable(I, (n, nnz), (indptr,
 * indices)) of Appendix A).  All three arrays are device pointers, borrowed for
 * the duration of the call, never written and never freed by the library.
 */
typedef struct {
  int32_t n_rows;
  int32_t n_cols;
  int64_t nnz;            /* must equal indptr[n_rows] and be < 2^31 */
  const int32_t* indptr;  /* device, [n_rows + 1], indptr[0] == 0, non-decreasing */
  const int32_t* indices; /* device, [nnz], strictly ascending inside a row, in [0, n_cols) */
  const float* values;    /* device, [nnz] */
} sptir_csr_t;

/* Opaque handle of a decomposed matrix; owns its device arrays. */
typedef struct sptir_hyb sptir_hyb_t;

/*
 * The flat hyb arrays, in the canonical layout that is compared bit for bit
 * with the CPU oracle.  B = c*(k+1) buckets, bucket id b = p*(k+1) + i for
 * partition p and width 2^i; empty buckets are kept.
 *   BUCKET_ROW_PTR  int64 [B+1]  prefix of ELL rows per bucket
 *   BUCKET_SLOT_PTR int64 [B+1]  prefix of stored slots per bucket (rows * 2^i)
 *   ELL_ROW         int32 [R]    row id of every ELL row, ascending inside a bucket
 *   ELL_COL         int32 [S]    global column ids, row-major inside a bucket
 *                                (slot = slot_ptr[b] + q*2^i + j, the flattening
 *                                rule of Section 3.4.1); a pad repeats the last
 *                                real column of its row piece
 *   ELL_VAL         float [S]    values in CSR order; pads are +0.0f
 *   REM_PART_PTR    int32 [c+1]  prefix of remainder pieces per partition
 *   REM_ROW         int32 [M]    row id of every remainder piece, ascending inside a partition
 *   REM_PTR         int64 [M+1]  prefix of piece lengths
 *   REM_COL         int32 [T]    global column ids
 *   REM_VAL         float [T]
 */
typedef enum {
  SPTIR_HYB_BUCKET_ROW_PTR = 0,
  SPTIR_HYB_BUCKET_SLOT_PTR = 1,
  SPTIR_HYB_ELL_ROW = 2,
  SPTIR_HYB_ELL_COL = 3,
  SPTIR_HYB_ELL_VAL = 4,
  SPTIR_HYB_REM_PART_PTR = 5,
  SPTIR_HYB_REM_ROW = 6,
  SPTIR_HYB_REM_PTR = 7,
  SPTIR_HYB_REM_COL = 8,
  SPTIR_HYB_REM_VAL = 9,
  SPTIR_HYB_N_ARRAYS = 10,
  /* What sptir_spmm reads instead of the canonical arrays (derived from them at build time; exported so that a
   * test can decode it and find every non-zero of A exactly once).  The chunk stream: fixed records of four
   * 64-slot chunks ("quads"), each [256 column words][256 values unless values_per_row][256 row words unless
   * compact_stream]; first the chunk lists, list (launch l, row block b) at chunks RB_CHUNK_PTR[l * n_row_blocks
   * + b] .. [.. + 1), then from chunk n_work_items on the heavy sequence, heavy list w at its chunks heavy_list_items * w ...
   * A compact column word holds the column relative to the first column of the launch in bits 0..19 (heavy
   * chunks: the column itself), bits 20..26 the row relative to the row block (heavy chunks: the slot at which a
   * piece ends in the chunk), bit 27 "the slot holds an entry", bits 28..30 the chunk kind (3: eight queues of
   * eight slots, slot 8q + j continuing queue q; 7: 64 slots of one row piece), bit 31 the hand-over flag (queue
   * chunk: this slot is the last entry of a row piece; otherwise the chunk's: a piece ends in it).  Without
   * compact_stream the column word is the column and the row word holds bits 0..15 row (or end slot), 16..21 kind
   * (3 or 31), bit 22 hand-over, bit 23 / the value -1 "no entry". */
  SPTIR_PLAN_STREAM = 100,            /* int32 */
  SPTIR_PLAN_RB_CHUNK_PTR = 101,      /* int64 [n_phases * n_row_blocks + 1] */
  SPTIR_PLAN_RB_ORDER = 102,          /* int32 [n_phases * n_row_blocks]: launch order of the row blocks */
  SPTIR_PLAN_HLIST_FIRST_SLOT = 103,  /* int32 [n_heavy_lists]: partial-sum row of each heavy list's first write */
  SPTIR_PLAN_ROW_SLOT_PTR = 104,      /* int32 [n_rows + 1] */
  SPTIR_PLAN_ROW_SLOTS = 105,         /* int32: the partial-sum rows that are added to row r of Y */
  SPTIR_PLAN_HEAVY_ROWS = 106,        /* int32: the rows with heavy pieces, ascending */
  SPTIR_PLAN_ROW_VAL = 107            /* float [n_rows], only with values_per_row */
} sptir_hyb_array_id;

typedef struct {
  int32_t n_rows, n_cols;
  int32_t n_col_parts;      /* c */
  int32_t max_bucket_log2;  /* k */
  int32_t part_width;       /* w = ceil(n_cols / c) */
  int32_t n_buckets;        /* B = c*(k+1) */
  int64_t nnz;              /* true non-zeros of A */
  int64_t n_ell_rows;       /* R */
  int64_t n_ell_slots;      /* S, pads included */
  int64_t n_pad_slots;      /* S + T - nnz */
  int64_t n_rem_pieces;     /* M */
  int64_t n_rem_nnz;        /* T */
  int64_t n_work_items;     /* 64-slot chunks of the chunk lists one sptir_spmm call walks (padding chunks included) */
  int32_t item_slots;       /* slots per chunk */
  int32_t row_block;        /* rows of Y one wavefront accumulates on chip */
  int32_t n_phases;         /* chunk-list launches per sweep when rounds == 0 (groups of column partitions) */
  int32_t rounds;           /* 1: every chunk list sweeps all column partitions and the lists run in rounds of as many
                               row blocks as the GPU holds at once (Y is written once); 0: one launch per group of
                               partitions, each adding to the Y of the one before */
  int64_t n_heavy_pieces;   /* row pieces with more than heavy_len real entries: summed by a launch of their own */
  int64_t n_heavy_items;    /* their 64-slot chunks */
  int64_t n_heavy_nnz;      /* their real entries */
  int32_t heavy_len;
  int32_t n_heavy_lists;    /* wavefronts of that launch per feature tile */
  int32_t values_per_row;   /* 1: every row of A has one value for all its entries and the SpMM stream holds none */
  int32_t compact_stream;   /* 1: 8-byte stream records (4 with values_per_row), 0: 12-byte (8) */
  int32_t n_row_blocks;
  int32_t parts_per_launch; /* column partitions one chunk list sweeps */
  int64_t device_bytes;     /* device memory the handle owns */
  int32_t full_rows;        /* 1: sptir_spmm uses feature tiles of 128 floats where feat and alignment allow */
  int32_t heavy_list_items; /* chunks per heavy list (16, fewer when the matrix has few heavy chunks) */
} sptir_hyb_info_t;

/*
 * Device allocator hook.  alloc(bytes, ctx, stream) returns a device pointer
 * aligned to at least 256 bytes, or NULL; free_(ptr, ctx) releases it.  The
 * default (both NULL) is hipMalloc / hipFree.  The hook is process-global and
 * must not be changed while a hyb object allocated through it is alive.
 */
typedef void* (*sptir_alloc_fn)(size_t bytes, void* ctx, void* stream);
typedef void (*sptir_free_fn)(void* ptr, void* ctx);
sptir_status_t sptir_set_allocator(sptir_alloc_fn alloc, sptir_free_fn free_, void* ctx);

/*
 * Under the default allocator sptir_hyb_build keeps the temporary device blocks of a call (at most 8 blocks and
 * 512 MB in all, none larger than 256 MB) for the next call instead of giving them back with hipFree, which costs more
 * than a whole small build.  This call frees what is being kept.  Handles are not affected.  With an allocator of
 * the caller's nothing is ever kept.
 */
sptir_status_t sptir_release_scratch(void);

/*
 * Format decomposition CSR -> hyb(c,k) on the GPU (Section 4.2.1 bucketing
 * rule; the "copy to the new format" step of Section 3.2.1 done once, as
 * pre-processing).  Runs a validation pass, a per-(row, partition) length
 * histogram, scans, and a stable scatter, all on `stream`
 * (a hipStream_t passed as void*; NULL is the default stream), and synchronises
 * that stream before returning.
 *   n_col_parts     c >= 1
 *   max_bucket_log2 0 <= k <= 30; ELL widths are 1, 2, ..., 2^k
 * On success *out receives a handle to release with sptir_hyb_destroy.
 * Errors: INVALID_ARG (null pointers, bad sizes, indptr not a non-decreasing
 * prefix ending at nnz), UNSORTED, OVERFLOW (nnz >= 2^31, or more than 2^31-1
 * ELL rows / remainder pieces), ALLOC, HIP.
 */
sptir_status_t sptir_hyb_build(const sptir_csr_t* csr, int32_t n_col_parts, int32_t max_bucket_log2,
                               void* stream, sptir_hyb_t** out);

/*
 * sptir_hyb_build with the choices spelled out that it otherwise makes from the sizes.  A zeroed struct (only
 * struct_size set) asks for the defaults; none of these fields changes the canonical arrays or, beyond float
 * rounding, the result of sptir_spmm.
 */
typedef struct {
  int32_t struct_size;        /* sizeof(sptir_build_options_t) */
  int32_t feat_hint;          /* feature size sptir_spmm will mostly run at (sizes the row blocks); 0: unknown */
  int32_t row_block;          /* rows of Y per wavefront: a power of two in 8..256; 0: chosen */
  int32_t parts_per_launch;   /* column partitions one chunk list sweeps; 0: chosen (n_col_parts when rounds) */
  int32_t rounds;             /* 0: chosen; 1: rounds (see sptir_hyb_info_t.rounds); 2: one launch per group of partitions */
  int32_t wide_stream;        /* 1: always 12-byte stream records */
  int32_t heavy_len;          /* row pieces with more real entries are summed by the heavy-piece launch; 0: chosen */
  int32_t sweep_kb;           /* kilobytes one sweep over the launches may touch: of Y without rounds (0: 163840),
                                 of X in rounds (0: 131072); wider operands are taken in groups of feature tiles */
  int32_t release_canonical;  /* 1: free ELL_COL, ELL_VAL, REM_COL and REM_VAL once the SpMM stream is packed
                                 (sptir_hyb_array then reports SPTIR_ERR_UNSUPPORTED for them) */
  int32_t no_spmm_plan;       /* 1: canonical arrays only; sptir_spmm refuses the handle */
  int32_t keep_values;        /* 1: the SpMM stream stores a value per entry even where every row of A has one
                                 value for all its entries (otherwise such a matrix is stored without values and
                                 the rows of Y are scaled at the end: half the stream bytes) */
  int32_t light_piece_len;    /* mean real length of the row pieces of at most 64 entries, if the caller knows it
                                 (sptir_hyb_build takes it from its histogram); 0: unknown, taken to be short.
                                 Rounds are chosen when it is below 16: Y round trips then cost more than the
                                 wavefronts of a round lose by drifting apart */
  int32_t full_rows;          /* 0: chosen; 1: a wavefront gathers whole 512-byte runs of a row of X (one feature
                                 tile of 128 floats, 32 lanes per entry) wherever feat is a multiple of 128, X and Y
                                 are 16-byte aligned and the row block has at most 64 rows, instead of one 128-byte line per entry and feature tile with
                                 the tiles bound to XCDs; 2: never.  Never chosen: it measured slower on every
                                 workload tried (the option stays so that the comparison can be repeated) */
} sptir_build_options_t;

sptir_status_t sptir_hyb_build_ex(const sptir_csr_t* csr, int32_t n_col_parts, int32_t max_bucket_log2,
                                  const sptir_build_options_t* options /* NULL: defaults */, void* stream,
                                  sptir_hyb_t** out);

/* The paper's rule of thumb for k (Section 4.2.1): ceil(log2(nnz / n_rows)), clamped to [0, 30]. */
int32_t sptir_default_bucket_log2(int64_t nnz, int32_t n_rows);

/*
 * Host-only query: 1 if the SpMM kernels may form the byte offset of a gathered row of X (column x feat x 4 + the
 * lane's offset inside the row) with the 24-bit multiply and 32-bit adds, for a launch whose columns span n_cols
 * and a feature size feat: both factors below 2^24 and the largest offset below 2^32.  0 otherwise (the kernels
 * then use 64-bit addresses), also for arguments that make no sense.  Exposed so that the rule can be tested
 * without a GPU.
 */
int32_t sptir_gather_offsets_fit_32(int64_t n_cols, int32_t feat);

/*
 * Format search (the tuning rule of Section 4.2.1: try several c, keep the
 * fastest).  Builds hyb(c, k) for every c of c_candidates (host array;
 * n_candidates == 0 selects the paper's {1, 2, 4, 8, 16}), runs sptir_spmm
 * `reps` times after one warm-up on zero-filled scratch operands of width
 * `feat`, and returns the decomposition with the smallest mean time.  The
 * launch plan of every candidate is sized for `feat` (feature sizes up to 64
 * get smaller row blocks than sptir_hyb_build chooses, so that a launch still
 * has enough wavefronts); the result serves any feat.
 *   max_bucket_log2  k for every candidate; negative selects sptir_default_bucket_log2
 *   best_c           receives the chosen c (may be NULL)
 *   ms_per_candidate host array [n_candidates] of mean milliseconds (may be NULL)
 * Allocates X and Y scratch (n_cols*feat and n_rows*feat floats) through the
 * allocator hook and synchronises `stream`.  Errors: those of sptir_hyb_build
 * and sptir_spmm; on error nothing is returned and nothing stays allocated.
 */
sptir_status_t sptir_hyb_search(const sptir_csr_t* csr, const int32_t* c_candidates, int32_t n_candidates,
                                int32_t max_bucket_log2, int32_t feat, int32_t reps, void* stream,
                                sptir_hyb_t** out, int32_t* best_c, float* ms_per_candidate);

/*
 * The launch plan that sptir_hyb_search (feat known) and sptir_spmm would choose for a matrix of these sizes:
 * host arithmetic only, no device is touched.  stored_slots is what the decomposition stores (ELL slots with
 * their pads plus remainder non-zeros; nnz is a fair stand-in).  Section 4.2.1 motivates column partitions by
 * the cache hit rate of X; on this GPU that decides how many partitions one launch may sweep, see
 * parts_per_launch.  X and Y are taken to be 16-byte aligned.
 */
typedef struct sptir_launch_plan {
  int32_t row_block;         /* rows of Y one wavefront keeps in LDS */
  int32_t parts_per_launch;  /* column partitions one chunk list sweeps */
  int32_t n_launches;        /* chunk-list launches per sweep when rounds == 0 */
  int32_t compact_stream;    /* 1: 8-byte records, 0: 12-byte records */
  int32_t n_feature_tiles;   /* tiles of 32 (16 for feat <= 16) floats that Y is cut into */
  int32_t tiles_per_sweep;   /* feature tiles one sweep over the launches covers */
  int32_t n_sweeps;
  int32_t rounds;            /* 1: the chunk lists run in rounds and Y is written once */
  int32_t full_rows;         /* 1: feature tiles of 128 floats (see sptir_build_options_t.full_rows) */
} sptir_launch_plan_t;

sptir_status_t sptir_launch_plan(int32_t n_rows, int32_t n_cols, int64_t stored_slots, int32_t n_col_parts,
                                 int32_t feat, const sptir_build_options_t* options /* NULL: defaults */,
                                 sptir_launch_plan_t* out);

/*
 * Y = A * X on the hyb decomposition (SpMM equation of Section 4.2.1; Y is
 * overwritten, rows without non-zeros become 0, as the init block of the
 * Appendix A script prescribes).
 *   X  device, [n_cols, feat] row-major float32, read only
 *   Y  device, [n_rows, feat] row-major float32, must not overlap X
 *   feat >= 1
 * Only enqueues work on `stream` (no synchronisation, no allocation).  The
 * chunk lists run in rounds (sptir_hyb_info_t.rounds: a launch per as many row
 * blocks as the GPU holds wavefronts, Y written once; an X wider than half the
 * memory-side cache is taken in sweeps of 128 or 256 feature columns, the heavy
 * pieces of a sweep right after its lists) or as one launch per group
 * of column partitions (n_phases launches, each adding to what the earlier ones
 * left in Y; a Y wider than the memory-side cache is then produced in several
 * such sweeps, each over a group of feature columns).  Heavy row pieces
 * (n_heavy_pieces > 0) take two more launches per 128 features (one where the
 * chunk lists are a single launch and the heavy lists the smaller part: they
 * then share that launch): their partial
 * sums pass through scratch memory that the handle owns, so calls on one handle
 * that has heavy pieces must not overlap in time.  No atomics are used and every
 * sum has a fixed order, so two calls with the same handle and X on the same GPU
 * give bit-identical Y.  The order differs from CSR order (sums are regrouped by
 * partition and bucket), so Y matches a CSR product only up to float rounding.  A
 * pad slot multiplies X by +0.0f: X must be finite.
 * Errors: INVALID_ARG, OVERFLOW (feat so large that the launch grid exceeds
 * 2^31 workgroups), HIP.
 */
sptir_status_t sptir_spmm(const sptir_hyb_t* hyb, const float* X, float* Y, int32_t feat, void* stream);

/*
 * Measurement aid: sptir_spmm with HIP events recorded on `stream` between its groups of launches, so that a
 * benchmark can price each kernel by the time it really took inside the call.  Synchronises `stream` before it
 * returns; creates and destroys a few events.  Same results as sptir_spmm.
 *   ms_lists   the chunk-list launches (k_spmm_hyb), n_list_launches of them
 *   ms_heavy   the heavy-piece launches (k_spmm_heavy)
 *   ms_reduce  the launches that add the heavy pieces' partial sums to Y (k_heavy_reduce)
 */
typedef struct {
  float ms_lists, ms_heavy, ms_reduce;
  int32_t n_list_launches, n_heavy_launches, n_reduce_launches;
} sptir_spmm_times_t;
sptir_status_t sptir_spmm_timed(const sptir_hyb_t* hyb, const float* X, float* Y, int32_t feat, void* stream,
                                sptir_spmm_times_t* out);

/*
 * The two on-chip roofs the SpMM kernels are priced against, measured on the current device (Section 4.2.1
 * names the cache hit rate of X as what column partitions buy; what a hit then costs is this gather rate).
 * sptir_roof_gather: every group of 8 lanes of n_workgroups x 4 wavefronts reads one 128-byte line (16 bytes a
 * lane, 8 loads in flight) of a random row of X[0 .. n_rows) (row_floats floats per row, 16-byte aligned),
 * iters x 8 times; `tiles` > 1 spreads the lines over that many 32-float feature tiles, bound to workgroup id
 * modulo 8 like the SpMM kernels bind tiles to XCDs.  *ms_out receives the time of one launch (after one
 * untimed launch), *bytes_out the bytes it gathered.  sptir_roof_fma: n_workgroups x 256 lanes issue iters x 8
 * independent float32 FMAs; *flops_out receives 2 flops per FMA.  `sink` is a device float the kernels may
 * write (they all but never do).  Both create two events and synchronise `stream`.
 */
sptir_status_t sptir_roof_gather(const float* X, int64_t n_rows, int32_t row_floats, int32_t tiles,
                                 int32_t n_workgroups, int32_t iters, float* sink, void* stream, float* ms_out,
                                 double* bytes_out);
sptir_status_t sptir_roof_fma(int32_t n_workgroups, int32_t iters, float* sink, void* stream, float* ms_out,
                              double* flops_out);

/*
 * sptir_spmm for callers that cannot allocate device memory or let a library do so: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * Y.  The one buffer sptir_spmm needs beyond its inputs and outputs, the partial sums of heavy row pieces
 * (sptir_hyb_info_t.n_heavy_pieces > 0; 128 floats for every heavy piece and every heavy list), does not come
 * from the handle here but from a static device array of SPTIR_NOALLOC_SCRATCH_BYTES inside the library, which
 * every GPU the library runs on holds until the process ends.  The call allocates and frees nothing, on any path.
 * A matrix whose partial sums do not fit ((n_heavy_pieces + n_heavy_lists) * 512 bytes exceed the array) is
 * refused with SPTIR_ERR_UNSUPPORTED before anything is enqueued, and sptir_last_hip_error() then says by how
 * much.  Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU race (also calls
 * on different handles and different streams); calls ordered by a stream or by the caller are fine.  Nothing in
 * the array has to start at zero: each call overwrites every element it later reads.
 */
#define SPTIR_NOALLOC_SCRATCH_BYTES (8u * 1024u * 1024u)
sptir_status_t sptir_spmm_noalloc(const sptir_hyb_t* hyb, const float* X, float* Y, int32_t feat, void* stream);

/*
 * Y = A * X straight from CSR, one pass, no decomposition: the "no-hyb"
 * variant that Section 4.2.1 compares hyb against.  Same argument meaning as
 * sptir_spmm; the CSR arrays are device pointers and are assumed valid (they
 * are not re-validated).  Only enqueues work on `stream`.
 */
sptir_status_t sptir_spmm_csr(const sptir_csr_t* csr, const float* X, float* Y, int32_t feat, void* stream);

/*
 * SDDMM on the structure of a CSR matrix (the SDDMM equation of Section 4.2):
 *     B[i,j] = A[i,j] * sum_k X[i,k] * Y[k,j]      for every stored (i,j) of A.
 * The paper does not fix how Y is laid out; this entry point takes its
 * transpose, so that both dense operands are read by rows:
 *   X         device, [n_rows, feat] row-major float32
 *   Yt        device, [n_cols, feat] row-major float32, Yt[j,k] = Y[k,j]
 *   B_values  device, [nnz] float32, parallel to csr->values (same row/column per position);
 *             may be csr->values itself, must not overlap anything else
 * The CSR arrays are device pointers and are assumed valid (not re-validated).
 * Only enqueues work on `stream`; no allocation.  Every entry is a fixed-order
 * sum, so results are reproducible bit for bit.
 * Errors: INVALID_ARG, OVERFLOW (nnz >= 2^31), HIP.
 */
sptir_status_t sptir_sddmm_csr(const sptir_csr_t* csr, const float* X, const float* Yt, float* B_values,
                               int32_t feat, void* stream);

/*
 * The same SDDMM with its entries visited in column-partition order, the way
 * Section 4.2.1 partitions columns for cache locality: a plan lists the entries
 * of every partition, each of the 8 XCDs sweeps its own partitions one after
 * the other, and the rows of Yt of one partition stay in that XCD's L2.  The
 * plan depends on the sparse structure only and is reused for any values, X,
 * Yt and feat.
 *   n_col_parts  number of column partitions; 0 chooses it from feat_hint (the
 *                feature size the plan will mostly run at) and the row lengths,
 *                and may settle for 1, which keeps CSR order
 *   csr->values  is not read (may be NULL); indptr / indices are device arrays,
 *                columns strictly ascending inside a row (UNSORTED if the pieces
 *                do not tile the rows)
 * The plan owns device memory of about 12 bytes per non-zero, obtained through
 * the allocator hook; sptir_sddmm_plan_build synchronises `stream`.
 */
typedef struct sptir_sddmm_plan sptir_sddmm_plan_t;

typedef struct {
  int32_t n_rows, n_cols;
  int32_t n_col_parts;  /* partitions in use (1: entries stay in CSR order) */
  int32_t part_width;
  int64_t nnz;
  int64_t n_runs;       /* runs of at most 512 entries, one wavefront each (0 when n_col_parts == 1) */
  int64_t device_bytes;
} sptir_sddmm_plan_info_t;

/*
 * The number of column partitions sptir_sddmm_plan_build chooses when it is passed n_col_parts == 0 (host
 * arithmetic only): a multiple of 8 such that one partition's rows of Yt (width * feat * 4 bytes) fit an XCD's
 * L2 and a (row, partition) piece still holds a few entries, or 1 (CSR order).  feat_hint 0 stands for 128.
 */
int32_t sptir_sddmm_default_col_parts(int32_t n_rows, int32_t n_cols, int64_t nnz, int32_t feat_hint);

sptir_status_t sptir_sddmm_plan_build(const sptir_csr_t* csr, int32_t n_col_parts, int32_t feat_hint, void* stream,
                                      sptir_sddmm_plan_t** out);
/* values, B_values: device [nnz] in CSR order (B_values may be values itself); X, Yt, feat as for sptir_sddmm_csr.
 * Only enqueues work on `stream`; no allocation; results are bit-reproducible. */
sptir_status_t sptir_sddmm(const sptir_sddmm_plan_t* plan, const float* values, const float* X, const float* Yt,
                           float* B_values, int32_t feat, void* stream);
sptir_status_t sptir_sddmm_plan_info(const sptir_sddmm_plan_t* plan, sptir_sddmm_plan_info_t* out);
sptir_status_t sptir_sddmm_plan_destroy(sptir_sddmm_plan_t* plan); /* NULL is accepted */

/*
 * Relational gather-matmul-scatter (RGMS equation of Section 4.4):
 *     Y[i,l] = sum_r sum_j sum_k A[r,i,j] * X[j,k] * W[r,k,l]
 * with A a 3-D sparse tensor of n_relations slices, each n_rows x n_cols.  As
 * in the paper, every slice is decomposed into hyb(1, k) buckets (k = 5 unless
 * given) and one fused kernel gathers rows of X, multiplies by W[r] on the
 * matrix cores and scatters into Y; X W[r] is never materialised.
 *   stacked   A as one CSR matrix of n_relations * n_rows rows and n_cols
 *             columns: stacked row r * n_rows + i holds A[r,i,:] (device arrays,
 *             int32 indices strictly ascending inside a stacked row, float32
 *             values; validated like sptir_hyb_build's input)
 *   max_bucket_log2   0..5, or negative for the paper's 5
 *   workspace_d_out   0, or a multiple of 32: the handle then also owns a scatter workspace of one row of
 *             workspace_d_out floats per (relation, row) pair, and sptir_rgms calls with d_out <= workspace_d_out
 *             (and a 16-byte aligned Y) store the product rows there and sum them per row of Y in a second pass,
 *             in a fixed order: results are then reproducible bit for bit, for about 20 % more time than the
 *             float atomics used otherwise.  This is not the n_relations x n_rows x d_out intermediate the
 *             paper avoids: it has one row per non-empty pair.
 * sptir_rgms_build owns device memory through the allocator hook and
 * synchronises `stream`.  Errors: those of sptir_hyb_build; INVALID_ARG if
 * stacked->n_rows is not a multiple of n_relations.
 */
typedef struct sptir_rgms_handle sptir_rgms_t;

typedef struct {
  int32_t n_relations, n_rows, n_cols, max_bucket_log2;
  int64_t nnz;
  int64_t n_stacked_rows_stored;  /* (relation, row) pairs with at least one entry, remainder pieces included */
  int64_t n_pad_slots;
  int64_t n_tiles;                /* 32-row tiles, one wavefront each */
  int32_t workspace_d_out;        /* widest d_out the scatter workspace serves (0: none) */
  int32_t reserved;
  int64_t device_bytes;
} sptir_rgms_info_t;

sptir_status_t sptir_rgms_build(const sptir_csr_t* stacked, int32_t n_relations, int32_t max_bucket_log2,
                                int32_t workspace_d_out, void* stream, sptir_rgms_t** out);
/*
 *   X  device, [n_cols, d_in] row-major float32, 16-byte aligned
 *   W  device, [n_relations, d_in, d_out] row-major float32
 *   Y  device, [n_rows, d_out] row-major float32, overwritten (rows without entries become 0)
 *   d_in in {32, 64, 128}, d_out a multiple of 32 (UNSUPPORTED otherwise; the paper runs 32 x 32)
 * Only enqueues work on `stream`; no allocation.  Products and sums are float32 (float32 matrix-core
 * instructions).  Without the workspace the contributions of different relations and buckets meet in Y through
 * float atomic adds in no fixed order, so results agree between runs to rounding, not bit for bit; with it only
 * pairs of more than 2^k entries still do.  Calls that share a handle's workspace must not overlap in time.
 * X must be finite (pad slots).
 */
sptir_status_t sptir_rgms(const sptir_rgms_t* rgms, const float* X, const float* W, float* Y, int32_t d_in,
                          int32_t d_out, void* stream);
sptir_status_t sptir_rgms_info(const sptir_rgms_t* rgms, sptir_rgms_info_t* out);
sptir_status_t sptir_rgms_destroy(sptir_rgms_t* rgms); /* NULL is accepted */

/* Releases the handle and its device arrays.  NULL is accepted. */
sptir_status_t sptir_hyb_destroy(sptir_hyb_t* hyb);

/* Fills *out with sizes and parameters of the decomposition. */
sptir_status_t sptir_hyb_info(const sptir_hyb_t* hyb, sptir_hyb_info_t* out);

/*
 * Borrowed device pointer and element count of one canonical array
 * (sptir_hyb_array_id); valid until sptir_hyb_destroy.  An empty array
 * reports *n_elems == 0 and may report a NULL pointer.
 */
sptir_status_t sptir_hyb_array(const sptir_hyb_t* hyb, int32_t which, const void** dev_ptr, int64_t* n_elems);

/* Static description of a status code. */
const char* sptir_status_string(sptir_status_t status);

/* Text of the last HIP error this thread saw inside the library ("" if none); also the reason of the last
 * SPTIR_ERR_UNSUPPORTED that sptir_spmm_noalloc returned on this thread. */
const char* sptir_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SPTIR_H_ */
