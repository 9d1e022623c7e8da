/*
 * emb_bag.h - C ABI of the MI355X (gfx950) multi-table EmbeddingBag forward.
 *
 * The operation is the embedding stage of DLRM inference as the paper states it (Sec. 2.1 and
 * Sec. 3.1, Algorithm 1): for every embedding table t and every sample b of a batch, the bag
 * (t, b) names "lookups per sample" rows of table t through an offsets array and an indices
 * array (the offsets -> indices -> table pointer chase of Sec. 3.1); the rows are gathered and
 * reduced element-wise into one vector of length ED, and table t's [BS, ED] result occupies
 * columns [t*D, t*D+D) of the output.  The paper launches one kernel per table, serially; this
 * library processes all tables of the batch in one call.
 *
 * Conventions
 *   - Pointers marked DEVICE are device (HBM) addresses valid on the current HIP device;
 *     pointers marked HOST are ordinary host addresses.  The library allocates and frees no
 *     device memory (its only device memory of its own is the fixed scratch array of
 *     emb_bag_profile_hot_rows_noalloc) and keeps no pointer after a call returns.
 *   - Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and never synchronise.
 *   - Every function returns an int status: EMB_OK (0) or a negative EMB_ERR_* code.  Nothing is
 *     thrown, printed or written to errno.
 *   - Results are deterministic: same inputs and same tuning give bit-identical output (fixed
 *     reduction order, no atomics in the forward path).
 */
#ifndef EMB_BAG_H_
#define EMB_BAG_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* table element types */
#define EMB_F32 0 /* IEEE binary32 rows */
#define EMB_F16 1 /* IEEE binary16 rows, widened exactly and accumulated in fp32 */
#define EMB_BF16 2 /* bfloat16 rows (upper half of a binary32), widened exactly, fp32 accumulation */
#define EMB_U8ROW 3 /* row-wise quantised rows: D unsigned 8-bit codes followed by an fp32 scale and
                       an fp32 bias (row = D + 8 bytes, which must be a multiple of 16 and at most
                       1024); element d of a row is scale * code_d + bias, accumulated in fp32 */
#define EMB_FP8ROW 4 /* the same row layout with 8-bit floating-point codes (OCP 8-bit floating
                        point, E4M3: bias 7, 3 fraction bits, subnormals, largest finite 448, no
                        infinities): element d is scale * e4m3(code_d) + bias.  The two NaN codes
                        (0x7F, 0xFF) give an unspecified result */

/* pooling modes: the two modes of the sum/mean kernel the paper studies (Sec. 3.1), and the
   element-wise maximum, the third pooling an embedding-bag operator usually offers */
#define EMB_SUM 0
#define EMB_MEAN 1 /* sum divided by the bag length; an empty bag gives 0 */
#define EMB_MAX 2  /* element-wise maximum over the bag's lookups that name an existing row; a bag
                      with none (empty, or invalid ids only) gives 0.  No per-sample weights.  The
                      result is an element of the table (exact) for fp32 / fp16 / bf16 rows; if a
                      gathered element is NaN the result for that output element is unspecified */

/* per-table access hints (one byte per table, see emb_bag_desc.table_hints) */
#define EMB_HINT_DEFAULT 0   /* rows are re-used within a batch: read them with the default cache
                                policy so that hot rows stay in L2 */
#define EMB_HINT_STREAMING 1 /* rows are (almost) never re-used within a batch: read them with the
                                non-temporal policy so that they do not occupy the caches */

/* status codes */
#define EMB_OK 0
#define EMB_ERR_NULL_PTR (-1)    /* a required pointer is NULL */
#define EMB_ERR_BAD_DIM (-2)     /* dim <= 0, row not a multiple of 16 bytes, bad out_ld, ... */
#define EMB_ERR_BAD_DTYPE (-3)   /* table_dtype is not one of the EMB_* element types */
#define EMB_ERR_BAD_MODE (-4)    /* mode is not EMB_SUM, EMB_MEAN or EMB_MAX */
#define EMB_ERR_UNSUPPORTED (-5) /* per-sample weights together with EMB_MEAN or EMB_MAX */
#define EMB_ERR_LAUNCH (-6)      /* the HIP runtime refused the launch */
#define EMB_ERR_BAD_SIZE (-7)    /* negative count, or a size beyond the supported range */
#define EMB_ERR_ALIGNMENT (-8)   /* tables / out not 16-byte aligned */
#define EMB_ERR_BAD_TUNING (-9)  /* unknown tuning key or value out of range */

/*
 * Launch tuning of one descriptor (HOST struct, read during the call only): the keys of
 * emb_bag_set_tuning as fields, with the same values and meanings (see there).  A descriptor
 * whose `tuning` pointer is set is planned from this struct and from nothing process-wide except
 * the tuning table (emb_bag_set_tuning_table, which fills the keys left automatic); one whose
 * pointer is NULL uses the process-wide keys.  Two models served by one process can so hold
 * different settings, and calls that carry their own tuning do not race with emb_bag_set_tuning.
 * A value out of range makes the call return EMB_ERR_BAD_TUNING.  Fill it with
 * emb_bag_tuning_defaults and change what differs.  No passage of the paper defines this struct;
 * the knobs are those of its Sec. 3.3, Sec. 4.2 and Sec. 7.
 */
typedef struct emb_bag_tuning {
  int32_t depth;            /* default 0 */
  int32_t addressing;       /* 0 */
  int32_t blocks_per_cu;    /* 0 */
  int32_t xcd_remap;        /* -1 */
  int32_t use_hints;        /* 1 */
  int32_t stream;           /* -1 */
  int32_t bags_per_group;   /* 0 */
  int32_t xcd_pieces;       /* 0 */
  int32_t per_table_launch; /* 0 */
  int32_t fuse;             /* 1 */
  int32_t bags_per_wave;    /* 0 */
  int32_t hot_split;        /* 0 */
  int32_t station;          /* 0 */
  int32_t reserved[3];      /* 0 */
} emb_bag_tuning;

/* Writes the defaults listed above (the settings of a fresh process); EMB_ERR_NULL_PTR for NULL. */
int emb_bag_tuning_defaults(emb_bag_tuning* tuning);

/*
 * Shape of one call (HOST struct, read during the call only).
 *
 *   T = num_tables, B = batch, D = dim.  Row size in bytes = D * sizeof(element) (D + 8 for the
 *   quantised types) must be a multiple of 16 and at most 65536 (1024 for the quantised types).
 *   Table t holds R_t = table_offsets[t+1] - table_offsets[t] rows, stored contiguously in one
 *   arena starting at arena row table_offsets[t]; D and the element type are the same for every
 *   table (the paper's tables are homogeneous, Sec. 5; see emb_bag_forward_mixed otherwise).
 */
typedef struct emb_bag_desc {
  int32_t num_tables;     /* T >= 1 */
  int32_t dim;            /* D >= 1 */
  int32_t table_dtype;    /* EMB_F32, EMB_F16, EMB_BF16, EMB_U8ROW or EMB_FP8ROW */
  int32_t mode;           /* EMB_SUM, EMB_MEAN or EMB_MAX */
  int64_t batch;          /* B >= 0; B == 0 is a no-op that returns EMB_OK */
  int64_t num_lookups;    /* NL = offsets[T*B]: entries in indices (and in per_sample_weights) */
  int64_t out_ld;         /* leading dimension of out, in floats; 0 means T*D; must be >= T*D
                             and a multiple of 4 */
  int64_t max_table_rows; /* an upper bound on max_t R_t, or 0 if unknown.  A bound that keeps
                             max_table_rows * row_bytes below 3.5 GiB lets the library use
                             32-bit buffer addressing; rows at or beyond the bound then read as
                             zero.  0 selects 64-bit addressing. */
  const uint8_t* table_hints; /* DEVICE, T bytes of EMB_HINT_*, or NULL (= all EMB_HINT_DEFAULT).
                             The paper profiles each table's access pattern offline and picks the
                             cache treatment from it (Sec. 4.3, Sec. 7 steps v-vi); this is where
                             that choice enters.  Hints change speed only, never results.
                             emb_bag_profile_reuse can produce them from a sample batch. */
  const float* table_avg_len; /* HOST, T floats, or NULL: the typical number of lookups per bag of
                             each table (a property of the feature: one-hot, multi-hot ...; e.g.
                             (offsets[(t+1)*B] - offsets[t*B]) / B of a sample batch).  Without
                             it one kernel serves all tables, chosen by the call's average
                             num_lookups / (T*B); with it, tables with short bags go to the
                             short-bag kernel and the others to the one-wavefront-per-bag kernel,
                             in two launches (see the "stream" tuning key).  Speed only. */
  const int64_t* hot_rows; /* DEVICE, int64 [T], or NULL: hot_rows[t] leading rows of table t are
                             its hot head, the rows a profile found to be looked up most often
                             (the paper finds the top 60K indices per table offline and keeps
                             their rows in L2, Sec. 4.3; emb_bag_profile_hot_rows finds them from
                             a sample batch).  The caller lays the table out with those rows
                             first and renumbers its row ids to match, once, offline.  gfx950
                             has no residency control to pin rows with; what the kernels can do
                             with the head is selected by the "hot_split" tuning key: regroup a
                             bag's lookups hot rows first, and read the hot rows with the
                             default cache policy and all others non-temporally so that the
                             stream of cold rows does not push the head out of L2 (hot_rows then
                             replaces table_hints: 0 = a streaming table, >= R_t = a table
                             re-used as a whole).  Measured on MI355X this lowers L2 misses but
                             not the time, so by default ("hot_split" 0) the field is not used.
                             Speed only: results change by summation order (rounding) at most.
                             Honoured by the one-wavefront-per-bag kernel with 32-bit buffer
                             addressing and a prefetch depth of 4 or 8 (plan->hot_split says
                             whether); ignored otherwise. */
  const emb_bag_tuning* tuning; /* HOST, or NULL (= the process-wide keys of emb_bag_set_tuning):
                             the launch tuning of this descriptor, see emb_bag_tuning */
} emb_bag_desc;

/*
 * emb_bag_forward - pooled lookup of all T*B bags (paper Sec. 3.1, Algorithm 1).
 *
 *   out[b*out_ld + t*D + d] = sum over j in [offsets[t*B+b], offsets[t*B+b+1]) of
 *                               w_j * table_t[indices[j]][d]            (w_j = 1 without weights)
 *   and that sum divided by the bag length in EMB_MEAN mode (0 for an empty bag); in EMB_MAX
 *   mode the maximum over the same j of table_t[indices[j]][d] instead (see EMB_MAX).
 *   Accumulation is in fp32; fp16 and bf16 rows are widened exactly first.
 *
 *   desc                HOST    shape, see above
 *   tables              DEVICE  arena [sum_t R_t, D] row-major, 16-byte aligned, f32 / f16 / bf16,
 *                               or [sum_t R_t, D + 8] bytes for EMB_U8ROW / EMB_FP8ROW
 *   table_offsets       DEVICE  int64 [T+1], first arena row of each table, non-decreasing
 *   indices             DEVICE  int64 [NL], table-local row ids, bags stored in (t, b) order
 *   offsets             DEVICE  int64 [T*B+1], CSR over bags: offsets[0] = 0, offsets[T*B] = NL
 *   per_sample_weights  DEVICE  float [NL] or NULL; only with EMB_SUM
 *   out                 DEVICE  float [B, out_ld], 16-byte aligned; columns [0, T*D) of every
 *                               row are overwritten (empty bags with +0.0f); no pre-zeroing
 *   stream              hipStream_t as void*; NULL = default stream
 *
 * Data-dependent errors cannot be reported by an asynchronous call; instead they are made
 * harmless: bag bounds are clamped to [0, NL] (a decreasing pair gives an empty bag) and a
 * lookup whose index is outside [0, R_t) contributes zero.  Use emb_bag_validate to count them.
 * Host-visible argument errors return a negative code and enqueue nothing.
 *
 * Size limits (EMB_ERR_BAD_SIZE beyond them): B < 2^31, and a launch holds at most 2^24 - 1
 * workgroups of four wavefronts, i.e. T * B * ceil(row bytes / 1024) <= 67,108,860 when every bag
 * has a wavefront of its own (fewer wavefronts are needed when the short-bag kernel serves the
 * call).  Split a larger batch over several calls.
 *
 * One call is one kernel launch.  With desc->table_avg_len the tables with short bags may be
 * served by the short-bag kernel and the others by the one-wavefront-per-bag kernel: as two
 * workgroup ranges of one fused launch (see the "fuse" tuning key), or - with more than 1024
 * tables, a prefetch depth other than 4 or 8, or "fuse" off - as two launches that write disjoint
 * columns and are enqueued on `stream` one after the other (emb_bag_plan_forward lists them).
 * More than 65535 tables are then served by one kernel.
 */
int emb_bag_forward(const emb_bag_desc* desc, const void* tables, const int64_t* table_offsets,
                    const int64_t* indices, const int64_t* offsets,
                    const float* per_sample_weights, float* out, void* stream);

/*
 * emb_bag_forward_mixed - the same pooled lookup for tables of DIFFERENT widths D_t.
 *
 *   The paper's tables are homogeneous (Sec. 5); production models mix widths.  Table t holds
 *   rows of D_t elements (row = D_t * sizeof(element) bytes, D_t + 8 for quantised rows; every row size
 *   a multiple of 16 and at most 1024 bytes) stored contiguously from BYTE offset
 *   table_byte_offsets[t] of the arena (R_t = (table_byte_offsets[t+1] - table_byte_offsets[t]) /
 *   row bytes), and its result occupies output columns [out_offsets[t], out_offsets[t+1]) with
 *   out_offsets[t+1] - out_offsets[t] = D_t.
 *
 *   desc                HOST    shape; desc->dims is a HOST array of the T widths, used to check
 *                               the call; the kernel itself reads the widths from out_offsets
 *   tables              DEVICE  arena bytes, 16-byte aligned; every table starts 16-byte aligned
 *   table_byte_offsets  DEVICE  int64 [T+1], non-decreasing
 *   out_offsets         DEVICE  int64 [T+1], out_offsets[0] >= 0, multiples of 4, last <= out_ld
 *   indices, offsets, per_sample_weights, out, stream   as in emb_bag_forward
 *
 * table_byte_offsets and out_offsets describe the model, not the batch, and are trusted the way
 * table_offsets is; a table whose entries contradict the rules above is skipped (nothing is
 * written for it).  Index and bag-bound defects are neutralised as in emb_bag_forward.
 *
 * One call is one kernel launch.  With short bags (see the "stream" tuning key) the tables are
 * grouped by row size (64, 128, 256, 512, 1024 bytes and below); every group the short-bag kernel
 * suits is served by that kernel and the other tables by the one-wavefront-per-bag kernel, as
 * consecutive workgroup ranges of one fused launch (see the "fuse" tuning key), or - with more
 * than 1024 tables, or "fuse" off - as launches of their own that write disjoint columns and are
 * enqueued on `stream` one after the other (emb_bag_plan_forward_mixed lists them).  More than
 * 65535 tables are refused in that case.
 */
typedef struct emb_bag_mixed_desc {
  int32_t num_tables;      /* T >= 1 */
  int32_t table_dtype;     /* EMB_F32 ... EMB_FP8ROW (one type for all tables) */
  int32_t mode;            /* EMB_SUM, EMB_MEAN or EMB_MAX */
  int32_t reserved;        /* 0 */
  int64_t batch;           /* B >= 0 */
  int64_t num_lookups;     /* NL = offsets[T*B] */
  int64_t out_ld;          /* leading dimension of out in floats; 0 means sum_t D_t */
  int64_t max_table_bytes; /* upper bound on the largest table in bytes, or 0 if unknown; a bound
                              below 3.5 GiB selects 32-bit buffer addressing */
  const int32_t* dims;     /* HOST, T widths D_t */
  const uint8_t* table_hints; /* DEVICE, T bytes of EMB_HINT_*, or NULL */
  const float* table_avg_len; /* HOST, T floats, or NULL: as in emb_bag_desc; decides per table
                              (instead of per call) which tables go to the short-bag kernel */
  const emb_bag_tuning* tuning; /* HOST, or NULL: as in emb_bag_desc */
} emb_bag_mixed_desc;

int emb_bag_forward_mixed(const emb_bag_mixed_desc* desc, const void* tables,
                          const int64_t* table_byte_offsets, const int64_t* out_offsets,
                          const int64_t* indices, const int64_t* offsets,
                          const float* per_sample_weights, float* out, void* stream);

/*
 * emb_bag_validate - count the data-dependent defects emb_bag_forward neutralises.
 *
 *   No passage of the paper defines this call: its inputs are traces that are well-formed by
 *   construction (Sec. 3.2, Sec. 5).  It checks the two arrays of the pointer chase of Sec. 3.1
 *   (offsets -> indices -> table) against the properties the forward call assumes.
 *
 *   Adds to *num_bad (DEVICE, one int64 that the caller has zeroed, on the same stream) one for
 *   every bag whose bounds are decreasing or outside [0, NL], one if offsets[0] != 0 or
 *   offsets[T*B] != NL, and one for every lookup whose index is outside [0, R_t).
 *   Same pointer meanings as emb_bag_forward; asynchronous on `stream`.  Only table_offsets'
 *   differences (the row counts R_t), num_tables, batch and num_lookups are used, so a batch for
 *   emb_bag_forward_mixed is checked with a descriptor of any valid dim and the cumulative row
 *   counts of its tables as table_offsets.
 */
int emb_bag_validate(const emb_bag_desc* desc, const int64_t* table_offsets,
                     const int64_t* indices, const int64_t* offsets, int64_t* num_bad,
                     void* stream);

/*
 * emb_bag_profile_reuse - measure how often each table's lookups repeat, and derive hints.
 *
 *   For every table t the first `window` lookups of the batch that go to t (fewer if the table
 *   receives fewer; window is clamped to [1, 16384]) are examined.  With n_t the number of
 *   lookups the whole batch sends to table t, w = window_used[t] and d = dup_count[t]:
 *     window_used[t] = number of lookups examined,
 *     dup_count[t]   = window_used[t] - (number of distinct row ids among them),
 *     hints[t]       = EMB_HINT_STREAMING if w == 0, or
 *                        w^2 * row_bytes * min(row_bytes, 128) > d * 2^36  (d repeats among w
 *                        draws put the rows in use at about w^2 / 2d; rows of 128 bytes or more
 *                        then exceed the 256 MiB memory-side cache, so a repeated row has left
 *                        it before it is asked for again; narrower rows share a 128-byte line
 *                        with 128 / row_bytes others and must exceed that many times the cache),
 *                        or
 *                        n_t * d * 1000 * 128 < threshold_permille * w^2 * min(row_bytes, 128)
 *                        (few of the table's lookups find their 128-byte cache line already
 *                        fetched: n_t draws over w^2 / 2d rows repeat a row in about
 *                        n_t * d / w^2 of cases, which for n_t <= window is the measured share
 *                        d / n_t itself, and a line holds 128 / row_bytes rows);
 *                      else EMB_HINT_DEFAULT.
 *   row_bytes follows from desc->dim and desc->table_dtype; all comparisons are exact integer
 *   arithmetic.  This is the device-side counterpart of the offline hot-index profiling of paper
 *   Sec. 4.3: uniform-random access (the paper's "random" dataset) over a table much larger
 *   than the batch shows practically no repeats, the power-law datasets show many, and so does
 *   a batch that draws a sizeable part of a small table.  Both constants are measured on MI355X
 *   (uniform tables, the hint forced either way): the streaming policy stops paying where about
 *   7.5 % of a table's lookups repeat a row, unless the rows in use outgrow the cache.
 *   threshold_permille < 0 selects the library default (75); values above 1,000,000 are taken
 *   as 1,000,000.
 *
 *   desc, indices, offsets   as in emb_bag_forward (desc->table_hints is ignored; num_tables,
 *                            batch, num_lookups and the row size matter; for tables of different
 *                            widths call once per width, or pass a typical dim)
 *   dup_count, window_used   DEVICE int32 [T] each, or NULL
 *   hints                    DEVICE uint8 [T], or NULL
 *   Asynchronous on `stream`; counts are exact and deterministic.
 */
int emb_bag_profile_reuse(const emb_bag_desc* desc, const int64_t* indices,
                          const int64_t* offsets, int32_t window, int32_t threshold_permille,
                          int32_t* dup_count, int32_t* window_used, uint8_t* hints, void* stream);

/*
 * emb_bag_profile_hot_rows - the k most frequently looked-up rows of every table in a sample batch.
 *
 *   The paper profiles offline to find "the top 60K hot indices" of each table and keeps their
 *   rows in L2 (Sec. 4.3); this is that profiling step on the device.  For every table t the
 *   first `window` lookups of the batch that go to t are examined (fewer if the table receives
 *   fewer); ids outside [0, 2^40 - 1) are not counted.  The distinct ids are ordered by
 *   (occurrences descending, id ascending) and the first k of them reported:
 *     num_hot[t]            = min(k, number of distinct ids examined),
 *     hot_ids[t*k + r]      = the r-th id of that order for r < num_hot[t], -1 beyond,
 *     hot_counts[t*k + r]   = its number of occurrences, 0 beyond.
 *   The result is unique (no two ids tie), exact and deterministic.  A caller that moves these
 *   rows to the front of table t, in this order, and renumbers its row ids accordingly can pass
 *   num_hot (widened to int64) as emb_bag_desc.hot_rows.
 *
 *   desc, indices, offsets   as in emb_bag_forward (only num_tables, batch and num_lookups
 *                            matter, so any valid dim serves)
 *   window                   1 .. 2^24 - 1 lookups examined per table
 *   k                        1 .. 65536
 *   hot_ids                  DEVICE int64 [T*k]
 *   hot_counts               DEVICE int32 [T*k]
 *   num_hot                  DEVICE int32 [T], or NULL
 *   workspace                DEVICE, 8-byte aligned, at least
 *                            emb_bag_profile_hot_rows_workspace(T, window, k) bytes: per table a
 *                            hash table of 2^ceil(log2(2*window)) 8-byte slots (at least 64) and a
 *                            sort buffer of 2^ceil(log2(k)) 8-byte keys (at least 2).  Its
 *                            contents on entry do not matter (the kernel clears what it uses) and
 *                            mean nothing afterwards; calls that share a workspace must not overlap
 *   workspace_bytes          size of the workspace; EMB_ERR_BAD_SIZE if too small
 *   Asynchronous on `stream`; one kernel launch, no allocation.
 *
 * emb_bag_profile_hot_rows_workspace returns the bytes needed, or EMB_ERR_BAD_SIZE (negative)
 * for arguments outside the ranges above.
 */
int64_t emb_bag_profile_hot_rows_workspace(int32_t num_tables, int64_t window, int64_t k);
int emb_bag_profile_hot_rows(const emb_bag_desc* desc, const int64_t* indices,
                             const int64_t* offsets, int64_t window, int64_t k, int64_t* hot_ids,
                             int32_t* hot_counts, int32_t* num_hot, void* workspace,
                             int64_t workspace_bytes, void* stream);

/*
 * emb_bag_profile_hot_rows_noalloc - emb_bag_profile_hot_rows for callers that cannot allocate
 * device memory and have no workspace to pass: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, results and errors, without the
 * workspace: the scratch memory is a fixed 16 MiB array in device memory that belongs to the
 * library (every GPU the library is used on holds it until the process ends).  The call
 * allocates and frees nothing; num_tables * (2^ceil(log2(2*window)) + 2^ceil(log2(k))) * 8
 * bytes (see emb_bag_profile_hot_rows_workspace) must not exceed 16,777,216, else
 * EMB_ERR_BAD_SIZE and nothing is enqueued.  All calls on one GPU share that array, which keeps
 * the previous call's contents (the kernel clears what it uses): calls that overlap in time on
 * one GPU, on different streams, race and give wrong results; calls on one stream are ordered.
 * The first call on a device looks the array's address up (hipGetSymbolAddress): make it
 * outside a graph capture.
 */
int emb_bag_profile_hot_rows_noalloc(const emb_bag_desc* desc, const int64_t* indices,
                                     const int64_t* offsets, int64_t window, int64_t k,
                                     int64_t* hot_ids, int32_t* hot_counts, int32_t* num_hot,
                                     void* stream);

/*
 * emb_bag_plan_forward / emb_bag_plan_forward_mixed - what the corresponding forward call would
 * launch for this descriptor under the current tuning, without launching anything: which kernel
 * (the paper's recipe of Sec. 7 picks a scheme per workload; this is where a caller sees the
 * pick), the prefetch depth, the grid and the block order.  Pure host code: no device pointer is
 * read, no HIP call is made, so it works on a machine without a GPU.
 *
 *   desc         HOST   as for the forward call (table_hints is only tested against NULL)
 *   has_weights  non-zero if the forward call would pass per_sample_weights
 *   plan         HOST   filled in; all zero for batch == 0
 *   which        which of the call's launches to describe, 0 .. num_launches - 1.
 *                       emb_bag_forward makes one launch, or two when desc->table_avg_len
 *                       separates tables with short bags from the others (the others are
 *                       listed first); emb_bag_forward_mixed
 *                       makes one stream-kernel launch per lanes-per-row class that kernel suits
 *                       and one wave-kernel launch for the other tables (as parts of one fused
 *                       launch when plan->fused is set)
 *   table_order  HOST   uint16 [min(T, 1024)] or NULL: the table at each of the launch's
 *                       plan->tables positions (the identity unless plan->listed)
 *   Returns the status the forward call would return for the descriptor alone
 *   (EMB_ERR_BAD_SIZE for a `which` beyond the last launch).
 *
 * Block order, when xcd_pieces > 0: workgroup g runs on XCD g % 8; with slot = g / 8,
 * unit = (slot / blocks_per_piece) * 8 + g % 8 is piece unit % xcd_pieces of the table at
 * position unit / xcd_pieces of the launch, and wavefront w of workgroup (slot % blocks_per_piece) of that
 * piece is wavefront (unit % xcd_pieces) * waves_per_piece + (slot % blocks_per_piece) * 4 + w
 * of the table if that number is below waves_per_piece within the piece and below
 * waves_per_table overall, and unit is below tables * xcd_pieces (otherwise it has no work).  With xcd_pieces == 0 wavefront
 * 4 * g + w of the grid is wavefront number 4 * g + w in position-major order.
 * In the wave kernel wavefront w of a table owns bags w * bags_per_wave .. (w + 1) * bags_per_wave
 * - 1 of it (one column slab of bag w / slabs when rows are longer than 1 KiB).
 */
#define EMB_KERNEL_WAVE 0   /* one wavefront per bag (per 1-KiB column slab of it) */
#define EMB_KERNEL_STREAM 1 /* short bags: a lane group streams consecutive bags */

typedef struct emb_bag_plan {
  int32_t kernel;            /* EMB_KERNEL_WAVE or EMB_KERNEL_STREAM */
  int32_t lanes_per_row;     /* 4..64; 0 = chosen per table (different widths) */
  int32_t depth;             /* row loads in flight per wavefront (per lane group: stream) */
  int32_t buffer_addressing; /* 1 = 32-bit buffer offsets with hardware range check, 0 = 64-bit */
  int32_t bags_per_group;    /* stream kernel: consecutive bags per lane group; else 0 */
  int32_t xcd_pieces;        /* pieces per table in XCD-affine order; 0 = natural order */
  int32_t listed;            /* 1 = the launch takes its tables from a list (see table_order):
                                a subset of the tables, or all of them dealt to XCDs by width */
  int32_t num_launches;      /* launches the forward call makes (1 unless tables of different
                                widths with short bags are split by lanes-per-row class) */
  int64_t grid_blocks;       /* 256-thread workgroups launched */
  int64_t wavefronts;        /* wavefronts that have work */
  int64_t waves_per_table;
  int64_t waves_per_piece;   /* XCD-affine order only */
  int64_t blocks_per_piece;  /* XCD-affine order only */
  int64_t tables;            /* tables (positions) this launch covers */
  int64_t fused;             /* 1 = the num_launches launches listed run as ONE kernel launch: they
                                are consecutive ranges of its workgroups, in the order listed,
                                each range padded to a multiple of 8 workgroups (see "fuse") */
  int64_t fused_grid_blocks; /* workgroups of that one launch; 0 unless fused */
  int32_t bags_per_wave;     /* wave kernel: consecutive bags of a table per wavefront (wavefront w
                                of a table owns bags w * bags_per_wave ...); else 0 */
  int32_t hot_split;         /* 1 = the launch honours desc->hot_rows */
  int32_t station;           /* 1 = row loads land in LDS (see "station"), 0 = in registers */
  int32_t reserved;          /* 0 */
} emb_bag_plan;

int emb_bag_plan_forward(const emb_bag_desc* desc, int has_weights, int32_t which,
                         emb_bag_plan* plan, uint16_t* table_order);
int emb_bag_plan_forward_mixed(const emb_bag_mixed_desc* desc, int has_weights, int32_t which,
                               emb_bag_plan* plan, uint16_t* table_order);

/*
 * emb_bag_set_tuning / emb_bag_get_tuning - process-wide launch tuning (the occupancy x
 * prefetch-depth search of paper Sec. 3.3, Sec. 4.2 and the recipe of Sec. 7, made a runtime
 * knob).  Keys (HOST strings):
 *   "depth"         row loads a wavefront keeps in flight: 1, 2, 4, 8 or 16; 0 = automatic
 *   "addressing"    0 = automatic (32-bit buffer addressing whenever the descriptor bounds the
 *                   largest table below 3.5 GiB, else 64-bit), 1 = force 64-bit global addressing
 *   "blocks_per_cu" cap on resident 256-thread workgroups per compute unit, 1..8; 0 = no cap
 *   "xcd_remap"     1 = XCD-affine order: a table's bags are dealt to one or two XCDs, so its hot
 *                   rows are fetched into one or two of the eight L2s instead of all eight
 *                   (the stand-in for the L2 pinning of Sec. 4.3); 0 = natural order;
 *                   -1 = automatic (on for large launches)
 *   "xcd_pieces"    pieces per table in the XCD-affine order: 1, 2, 4 or 8; 0 = automatic (the
 *                   smallest power of two that gives every XCD the same number of pieces)
 *   "per_table_launch" 1 = emb_bag_forward makes one launch per table, one after the other, the
 *                   launch structure of the paper's system (Sec. 3.1); for comparisons only.
 *                   0 (default) = all tables in one launch
 *   "use_hints"     1 (default) = honour desc->table_hints, 0 = ignore them
 *   "stream"        the kernel for short bags, in which a lane group streams several consecutive
 *                   bags so that row loads stay in flight across bag boundaries (the prefetch of
 *                   Sec. 4.2 carried over the bounds -> indices -> rows chain of Sec. 3.1):
 *                   -1 = automatic (average bag length num_lookups / (T * batch) below three
 *                   load instructions' worth of rows, i.e. 3 * 1024 / row bytes rounded to a
 *                   power of two: 24 at 128-byte rows, 12 at 256, 6 at 512, 3 at 1 KiB; rows of
 *                   at most 1 KiB; every pooling mode; either addressing), 0 = never, 1 =
 *                   whenever the row size allows it.  It adds a bag's rows in the order of its lookups; the
 *                   one-wavefront-per-bag kernel keeps several partial sums, so the two agree
 *                   to rounding, not to the bit.
 *                   With desc->table_avg_len the automatic choice is made per table.
 *   "bags_per_group" consecutive bags per lane group in that kernel, 1..63; 0 = automatic
 *   "fuse"          1 (default) = when a forward call would make several launches, they
 *                   become consecutive workgroup ranges of one launch (same results, bit for
 *                   bit; no ramp and drain per launch, which dominates at inference batch
 *                   sizes); possible when the launches' table lists hold at most 1024 tables
 *                   together (and, for emb_bag_forward, the depth is 4 or 8), for sum and mean
 *                   pooling (with or without weights); EMB_MAX calls keep their launches.
 *                   0 = separate launches
 *   "bags_per_wave" consecutive bags of a table that one wavefront of the one-wavefront-per-bag
 *                   kernel takes, 1..32; 0 = automatic (more for short bags, 1 for rows beyond
 *                   1 KiB).  The bounds of a wavefront's bags come with one load and the next
 *                   bag's row ids are requested while the current bag's rows are gathered (the
 *                   index prefetch of Sec. 4.2, run across bags).  Same results, bit for bit
 *   "hot_split"     what the kernels do with desc->hot_rows: 0 (default) = nothing; 1 = a bag's
 *                   lookups are regrouped hot rows first, hot rows read with the default cache
 *                   policy, all others non-temporally; 2 = regrouped only, one policy
 *   "station"       where the rows a wavefront has in flight land (the prefetch station of
 *                   Sec. 4.2): 0 (default) = in registers; 1 = in LDS (the paper's shared-memory
 *                   prefetch: `depth` slots of 1 KiB per wavefront, read back when the load has
 *                   landed), for the one-wavefront-per-bag kernel with buffer addressing, sum or
 *                   mean pooling without weights, depth 4 or 8 and no hot / cold split;
 *                   elsewhere, and in fused launches, the key is ignored (plan->station says
 *                   what a launch does).  Same results, bit for bit.  Measured on MI355X it is
 *                   never faster (a CU's registers hold more rows in flight than its LDS)
 * Not thread-safe against concurrent emb_bag_forward calls whose descriptor has no tuning of its
 * own (emb_bag_desc.tuning).
 */
int emb_bag_set_tuning(const char* key, int64_t value);
int emb_bag_get_tuning(const char* key, int64_t* value);

/*
 * emb_bag_set_tuning_table - per-shape tuning found by a sweep (the outcome of the paper's
 * profiling recipe, Sec. 7 steps ii-vii: multithreading level, prefetch distance and scheme per
 * workload; python -m paper_2410_22249_amd.autotune --table writes one).  Entry i covers calls
 * whose rows are at most max_row_bytes bytes (the widest row of emb_bag_forward_mixed) and whose
 * average bag length num_lookups / (T * batch) is at most max_avg_len; the FIRST entry that
 * covers a call supplies the keys that emb_bag_set_tuning has left at their automatic value
 * (depth 0, bags_per_wave 0, stream -1, bags_per_group 0); a key set there explicitly wins.
 * The library keeps its own copy of at most 64 entries; n = 0 clears the table.  HOST pointer.
 * Results never depend on the table (speed only; the short-bag kernel rounds differently from the
 * one-wavefront-per-bag kernel, see "stream").  Not thread-safe against concurrent forward calls.
 */
typedef struct emb_bag_tuning_entry {
  int32_t max_row_bytes;  /* >= 16 */
  float max_avg_len;      /* >= 0 */
  int32_t depth;          /* 0 (automatic), 1, 2, 4, 8 or 16 */
  int32_t bags_per_wave;  /* 0 (automatic) .. 32 */
  int32_t stream;         /* -1 (automatic), 0 or 1 */
  int32_t bags_per_group; /* 0 (automatic) .. 63 */
} emb_bag_tuning_entry;
int emb_bag_set_tuning_table(const emb_bag_tuning_entry* entries, int32_t n);

/* Static, NUL-terminated description of a status code (never NULL).  Library plumbing: no
   passage of the paper stands behind it. */
const char* emb_bag_status_string(int status);

/* Library version: major*10000 + minor*100 + patch.  Library plumbing, as above. */
int emb_bag_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EMB_BAG_H_ */
