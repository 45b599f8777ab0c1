/*
 * libtagc -- the per-GPU hot path of TAGC (Transformer-Aware Gradient
 * Compression, arXiv 2504.05638) for AMD MI355X (gfx950).
 *
 * One call sequence processes one gradient bucket (what one FSDP
 * communication hook sees, Algorithm 1) for N ranks simulated on one GPU:
 *
 *   tagc_plan            host only, once per bucket shape
 *   tagc_plan_upload     copies the segment table to the device, once
 *   for each rank r:  tagc_compress(PHASE_INDEX)    sparsify + create_index
 *   tagc_aggregate(PHASE_INDEX)                     All-Reduce(index) as OR (or add)
 *   for each rank r:  tagc_compress(PHASE_SKETCH)   compress -> Count Sketch
 *   tagc_aggregate(PHASE_SKETCH)                    Reduce as element-wise sum
 *   tagc_decompress                                 peeling_decompress
 *
 * Conventions for every function below
 *   - returns TAGC_OK (0) or a negative tagc_error; never throws;
 *   - "dev" pointers are device (HBM) addresses owned by the caller, "host"
 *     pointers are ordinary host memory; the library never allocates or frees
 *     device memory and never synchronises a stream;
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream); all
 *     device work of a call is enqueued on it, in order;
 *   - device buffers must be 16-byte aligned and at least as large as
 *     tagc_plan_sizes reports; their contents on entry do not matter unless
 *     stated;
 *   - argument errors are reported by return code before anything is
 *     enqueued; data-dependent conditions (peeling left a residue, non-finite
 *     inputs) are reported in device-side status words that the caller reads
 *     after synchronising.
 */
#ifndef TAGC_H
#define TAGC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tagc_error {
    TAGC_OK = 0,
    TAGC_EINVAL = -1,       /* bad argument (null pointer, misaligned, bad enum) */
    TAGC_ESIZE = -2,        /* a size exceeds what the format can address        */
    TAGC_EUNSUPPORTED = -3, /* valid request this build does not implement       */
    TAGC_EHIP = -4,         /* a HIP runtime call failed                         */
    TAGC_ENOMEM = -5        /* host allocation failed                            */
} tagc_error;

enum { TAGC_F32 = 0, TAGC_BF16 = 1 };                      /* tagc_config.dtype  */
enum { TAGC_SIZE_LOAD_FACTOR = 0, TAGC_SIZE_FIXED_RATIO = 1 }; /* .sizing        */
enum { TAGC_INDEX_OR1 = 0, TAGC_INDEX_ADD1 = 1, TAGC_INDEX_ADD4 = 2 }; /* .index_mode */
enum { TAGC_PHASE_INDEX = 1, TAGC_PHASE_SKETCH = 2 };
#define TAGC_SEG_COMPRESS 1u

/*
 * One layer (or layer shard) of the bucket.  Layer-selective compression
 * (section 3.2, "Selective Compressing"): segments without TAGC_SEG_COMPRESS
 * are neither read nor written and get no index bits and no sketch cells.
 * Compressed segments are renumbered, in table order, into one "c-index"
 * space; each segment's c-offset is rounded up to a multiple of 32.
 */
typedef struct tagc_segment {
    uint64_t offset;   /* element offset inside each rank's gradient buffer   */
    uint64_t length;   /* n_l, elements; < 2^31                                */
    uint32_t keep_ppm; /* survivors per million, i.e. (1 - theta) * 10^6; the */
                       /* segment keeps k_l = floor(n_l*keep_ppm/10^6) entries */
                       /* (section 3.2: at least theta of the values become 0) */
    uint32_t flags;    /* TAGC_SEG_COMPRESS or 0                               */
} tagc_segment;

typedef struct tagc_config {
    uint32_t dtype;         /* TAGC_F32 | TAGC_BF16: element type of the gradient */
    uint32_t n_ranks;       /* N, upper bound on ranks aggregated (sizing only)   */
    uint32_t n_hash;        /* must be 3                                          */
    uint32_t sizing;        /* TAGC_SIZE_LOAD_FACTOR: cells = sizing_milli/1000 x
                               non-zeros of the merged Index;
                               TAGC_SIZE_FIXED_RATIO: cells = n / (sizing_milli/
                               1000), the "c-x compression" of Table 1          */
    uint32_t sizing_milli;
    uint32_t index_mode;    /* TAGC_INDEX_OR1: 1 bit per parameter, merged by OR
                               (section 2.2).  TAGC_INDEX_ADD1 / TAGC_INDEX_ADD4:
                               the OR simulated by addition as over NCCL (same
                               section), see "Index modes" below                */
    uint32_t part_unknowns; /* max non-zeros per sketch partition, 0 = default  */
    uint32_t part_cells;    /* max cells per sketch partition (multiple of 3),
                               0 = default                                      */
    uint64_t seed;          /* hash seed; all ranks must use the same           */
    uint32_t decode_mode;   /* TAGC_DECODE_*; 0 = peeling only                  */
    uint32_t cell_type;     /* TAGC_CELL_*: what a cell of a rank's sketch is on
                               the wire; 0 = float32                            */
    uint32_t decode_workgroups; /* most workgroups the peeling kernel of
                               tagc_decompress runs at once; 0 = one per compute
                               unit.  A peeling workgroup needs a compute unit's
                               whole local memory, so a caller that keeps other
                               buckets' work in flight on other streams leaves
                               the rest of the device to them with a value
                               like a quarter of the compute units.  Results
                               and buffer sizes do not depend on it: plans that
                               differ in nothing else work on the same buffers  */
    uint32_t reserved;      /* must be 0                                        */
} tagc_config;

/*
 * Section 5 names quantised communication as the step beyond the float32-only
 * implementation.  TAGC_CELL_BF16: a rank builds its Count Sketch in float32
 * as always and rounds each cell to the nearest bfloat16 (ties to even) when
 * it writes rank->sketch, which then holds 16-bit cells; PHASE_SKETCH of
 * tagc_aggregate widens them and adds in float32 in rank order; the summed
 * sketch and everything after it stay float32.  Halves the sketch's volume;
 * decoded values carry the rounding noise of the cells they passed through
 * (lossless only when the cells are bfloat16 numbers anyway).
 */
#define TAGC_CELL_F32 0u
#define TAGC_CELL_BF16 1u

/*
 * Index modes (section 2.2).  The paper's implementation cannot OR over NCCL
 * and adds instead, on a 1-bit Index (fast, collides) or a 4-bit one (stable,
 * four times bigger); no layout is given.  Here the wire Index is an array of
 * unsigned 32-bit words that the aggregation adds as such (wrapping; a carry
 * runs into the next parameter's field, the carry out of a word is lost):
 *   TAGC_INDEX_ADD1  wire Index = local Index (parameter j = bit j&31 of word
 *                    j>>5); a position kept by an even number of ranks drops
 *                    out of the merged Index and its carries flip higher ones;
 *   TAGC_INDEX_ADD4  one 4-bit counter per parameter, parameter j in bits
 *                    4*(j&7).. of word j>>3 (4 * bitmap_words words per rank,
 *                    what tagc_rank_buffers.bitmap then holds); merged bit j =
 *                    counter j of the sum != 0: the OR for up to 15 ranks.
 * The merged Index stays 1 bit per parameter in both.  PHASE_SKETCH then
 * encodes only the pairs whose position the merged Index names, so that the
 * decoder's unknowns are exactly what the cells hold: a position a carry
 * erased is lost, one a carry invented decodes to 0.
 */

/* What tagc_decompress does with the summed sketch (section 2.2 names the two
 * decompression algorithms, peeling and estimation; the latter is a Count
 * Sketch point query: the median of an entry's three signed cell readings). */
#define TAGC_DECODE_PEEL 0u          /* peel; what cannot be recovered is 0       */
#define TAGC_DECODE_PEEL_ESTIMATE 1u /* peel; the rest is estimated from the cells
                                        as peeling left them (everything recovered
                                        already subtracted)                       */
#define TAGC_DECODE_ESTIMATE 2u      /* no peeling: every entry is estimated from
                                        the summed sketch as it is                */

typedef struct tagc_plan_s tagc_plan_t; /* opaque, host memory, immutable */

/* Every size a caller needs; bytes unless the name says otherwise. */
typedef struct tagc_sizes {
    uint64_t n_seg_compressed;
    uint64_t n_real;            /* sum of n_l over compressed segments          */
    uint64_t n_c;               /* size of the c-index space (padded, % 32 == 0) */
    uint64_t bitmap_words;      /* n_c / 32                                     */
    uint64_t pair_capacity;     /* K = sum of k_l: most pairs one rank emits    */
    uint64_t union_capacity;    /* most non-zeros the merged Index can have     */
    uint64_t partition_capacity;/* most sketch partitions                       */
    uint64_t sketch_cells_capacity; /* most sketch cells m                      */
    uint64_t part_unknowns, part_cells; /* format parameters in effect          */
    uint64_t grad_elems;        /* elements each rank's gradient buffer must hold
                                   (largest offset + length over compressed segments) */

    uint64_t table_bytes;       /* device copy of the segment table             */
    /* per rank */
    uint64_t rank_idx_bytes, rank_val_bytes, rank_cnt_bytes, rank_bitmap_bytes,
        rank_sketch_bytes, rank_workspace_bytes;
    /* shared (one per bucket) */
    uint64_t shared_bitmap_bytes, shared_sketch_bytes, shared_header_bytes,
        shared_bounds_bytes, shared_workspace_bytes, shared_status_bytes;
    /* decoder outputs */
    uint64_t out_idx_bytes, out_val_bytes, out_dense_bytes;

    /* Bits per parameter per rank on the wire (Figures 1 and 2): Index moved
     * by All-Reduce (payload counted twice), Count Sketch by Reduce (once).
     * In load-factor mode the sketch term uses sketch_cells_capacity. */
    double wire_index_bits, wire_sketch_bits, wire_total_bits;
} tagc_sizes;

/* rank `cnt` words (uint32) */
enum {
    TAGC_CNT_TOTAL = 0,     /* pairs emitted by this rank                        */
    TAGC_CNT_NONFINITE = 1, /* inputs with all-ones exponent seen (result then
                               unspecified but memory-safe)                      */
    TAGC_CNT_FLAGS = 2,     /* TAGC_FLAG_* bits                                  */
    TAGC_CNT_DENSE = 3,     /* segments that took the dense route (diagnostic)    */
    TAGC_CNT_RESERVED = 4,  /* 0                                                 */
    TAGC_CNT_SEG0 = 5       /* [5 + l] = pairs of compressed segment l           */
};
/* Behind the counts (rank_cnt_bytes covers it) tagc_aggregate(PHASE_INDEX) leaves,
 * for every rank it is given, the A + 1 positions at which that rank's sorted
 * pair list crosses the partition bounds; PHASE_SKETCH reads them. */
/* shared `header` words (uint32), written by tagc_aggregate(PHASE_INDEX) */
enum {
    TAGC_HDR_U = 0,       /* non-zeros of the merged Index                       */
    TAGC_HDR_A = 1,       /* sketch partitions                                   */
    TAGC_HDR_MSUB = 2,    /* cells per hash function per partition               */
    TAGC_HDR_M = 3,       /* total cells m = 3 * A * m_sub                       */
    TAGC_HDR_WORDS = 8
};
/* shared `status` words (uint32), written by tagc_decompress */
enum {
    TAGC_ST_UNRESOLVED = 0, /* non-zeros peeling did not recover (value 0, or an
                               estimate if the plan's decode mode asks for one)  */
    TAGC_ST_ROUNDS = 1,     /* peeling rounds of the slowest partition           */
    TAGC_ST_FLAGS = 2,      /* TAGC_FLAG_* bits                                  */
    TAGC_ST_ESTIMATED = 3,  /* entries whose value is an estimate                */
    TAGC_ST_WORDS = 8
};
#define TAGC_FLAG_OVERFLOW 2u   /* a capacity was exceeded: results invalid          */

/* Device buffers of one simulated rank (all dev, caller-owned). */
typedef struct tagc_rank_buffers {
    uint32_t *idx;      /* [pair_capacity] c-indices of survivors, ascending    */
    float *val;         /* [pair_capacity] their values widened to float32      */
    uint32_t *cnt;      /* [rank_cnt_bytes / 4] see TAGC_CNT_*                  */
    uint32_t *bitmap;   /* [rank_bitmap_bytes / 4] local Index as it goes on the
                           wire: bit j in word j>>5, bit j&31 (bitmap_words
                           words), or 4-bit counters with TAGC_INDEX_ADD4       */
    float *sketch;      /* [rank_sketch_bytes] local Count Sketch; cells
                           [0, m) are written, the rest untouched.  16-bit
                           cells with TAGC_CELL_BF16.  rank_sketch_bytes covers
                           sketch_cells_capacity cells of the plan's cell type
                           and, for float32 cells, 48 KiB behind them that
                           tagc_reduce_decompress may read (never use)         */
    void *workspace;    /* [rank_workspace_bytes] scratch, may be shared by ranks
                           processed one after another on one stream           */
    void *acc;          /* NULL, or [grad_elems] of the plan's dtype: the rank's
                           gradient accumulator (Algorithm 1: acc in, acc_next
                           out, in place).  Together with `bitmap` it is the
                           rank's error-feedback state: zero both before the
                           first step and keep both between steps; see
                           PHASE_INDEX                                          */
} tagc_rank_buffers;

/* Device buffers shared by the bucket (all dev, caller-owned). */
typedef struct tagc_shared_buffers {
    const void *table;  /* [table_bytes] filled by tagc_plan_upload and from then
                           on written by the library only: behind the segment
                           rows PHASE_INDEX keeps the plan's device state there
                           (one pre-threshold per segment, carried from call to
                           call as a speed hint that results never depend on;
                           counters and candidate histograms that every call
                           leaves at zero again).  PHASE_INDEX calls that share
                           a table must not overlap in time                    */
    uint32_t *bitmap;   /* [bitmap_words] merged Index                          */
    float *sketch;      /* [sketch_cells_capacity] summed Count Sketch          */
    uint32_t *header;   /* [TAGC_HDR_WORDS]                                     */
    uint32_t *bounds;   /* [shared_bounds_bytes / 4] first c-index of each partition
                           (A + 1 words, the last one n_c), then, from word
                           partition_capacity + 1 on, the partitions' hash
                           salts (A words), see tagc_aggregate             */
    void *workspace;    /* [shared_workspace_bytes]                             */
    uint32_t *status;   /* [TAGC_ST_WORDS]                                      */
} tagc_shared_buffers;

/*
 * Builds the host-side plan of a bucket: c-offsets, keep counts k_l, tile
 * decomposition, capacities and byte accounting (Algorithm 1's inputs theta
 * and the layer selection of section 3.2 become the segment table).
 * `segments` (host) is copied.  Errors: TAGC_EINVAL (null pointers, unknown
 * enum, n_hash != 3, n_ranks == 0, sizing_milli == 0, keep_ppm > 10^6,
 * part_cells not a multiple of 3 or too large for LDS), TAGC_ESIZE (a
 * segment of 2^31 elements or more, c-index space or sketch of 2^32 or more),
 * TAGC_ENOMEM.  *out is owned by the caller: tagc_plan_destroy.
 */
int tagc_plan(const tagc_config *config, const tagc_segment *segments,
              uint32_t n_seg, tagc_plan_t **out);
void tagc_plan_destroy(tagc_plan_t *plan);

/* Fills *out (host).  Never touches the device. */
int tagc_plan_sizes(const tagc_plan_t *plan, tagc_sizes *out);

/* Copies the plan's segment table into `table_dev` (table_bytes) on `stream` and
 * clears the device state behind it; the first PHASE_INDEX call on the plan
 * after an upload also samples pre-thresholds.  The plan must outlive the copy. */
int tagc_plan_upload(const tagc_plan_t *plan, void *table_dev, void *stream);

/*
 * PHASE_INDEX  (Algorithm 1: sparsify, create_index; threshold rule of
 *   section 3.2).  Reads `grad_dev` (dev, dtype of the plan, only the
 *   compressed segments).  For every compressed segment keeps the k_l entries
 *   of largest magnitude, ties to the lower position, exact zeros never; writes
 *   the survivors as (c-index, float32 value) pairs in ascending c-index to
 *   rank->idx / rank->val, counts to rank->cnt, and the local Index to
 *   rank->bitmap (every word is written).  Uses rank->workspace and the device
 *   state in shared->table (see tagc_shared_buffers).
 *   With rank->acc set (Algorithm 1, lines 1-2; section 3.2, local gradient
 *   accumulation) the entries of the compressed segments are first replaced by
 *   grad + acc, added in the gradient's own type (bf16: one float32 add rounded
 *   to nearest-even), and afterwards acc_next is, in those segments, that sum
 *   where the entry was not selected and zero where it was: what was selected
 *   plus acc_next is the sum, element by element.  grad_dev is only read.
 *   acc_next is left in two parts: rank->acc holds the sums everywhere, and
 *   rank->bitmap, the rank's new Index, names the entries that read as zero.
 *   The call reads acc through the Index the rank's previous call left in
 *   rank->bitmap in the same way (so rank->bitmap is an input too: all zero
 *   before the first step), then overwrites both.  Clearing the ~1 % selected
 *   entries in acc itself would cost a second pass over half of its cache
 *   lines; tagc_feedback_apply does it for a caller who wants the plain array.
 * PHASE_SKETCH (Algorithm 1: compress(g_shard, index)).  Needs the shared
 *   header written by tagc_aggregate(PHASE_INDEX), which must have been given
 *   this rank among its `ranks` (it leaves the rank's partition ranges in
 *   rank->cnt), and this rank's pairs; hashes every pair with the three hash
 *   functions into the rank's
 *   Count Sketch, cells [0, m) of rank->sketch (all of them are written).
 * Both phases read shared->table.
 */
int tagc_compress(const tagc_plan_t *plan, uint32_t phase, const void *grad_dev,
                  const tagc_rank_buffers *rank,
                  const tagc_shared_buffers *shared, void *stream);

/*
 * tagc_compress for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and errors as
 * tagc_compress, except that rank->workspace is ignored (it may be NULL):
 * PHASE_INDEX works on an array of TAGC_STATIC_WORKSPACE_BYTES that is part
 * of the library's device code, one copy per GPU, held until the process
 * ends.  Returns TAGC_ESIZE, before anything is enqueued, when the plan's
 * rank_workspace_bytes exceed that size.  The call allocates nothing (no
 * hipMalloc / hipFree, no allocating library routine); its first call on a
 * device looks the array's address up (do that call outside a graph capture).
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams, threads or plans) race, exactly like
 * tagc_compress calls sharing one rank->workspace.  The array keeps the last
 * call's contents; PHASE_INDEX clears what it needs clear, as it does for a
 * caller's workspace.
 */
#define TAGC_STATIC_WORKSPACE_BYTES (16u << 20)
int tagc_compress_static(const tagc_plan_t *plan, uint32_t phase, const void *grad_dev,
                         const tagc_rank_buffers *rank,
                         const tagc_shared_buffers *shared, void *stream);

/*
 * Error feedback, optional: clears in rank->acc the entries that rank->bitmap
 * names, after which rank->acc alone is acc_next of Algorithm 1 (line 2).  For
 * inspection and checkpoints; idempotent, and the following PHASE_INDEX call
 * gives the same results with or without it.  Needs rank->acc, rank->bitmap as
 * the rank's last PHASE_INDEX call left them, and shared->table.
 */
int tagc_feedback_apply(const tagc_plan_t *plan, const tagc_rank_buffers *rank,
                        const tagc_shared_buffers *shared, void *stream);

/*
 * Stands in for the two collectives of Algorithm 1 on one GPU.
 * PHASE_INDEX : shared->bitmap = OR over ranks[r].bitmap (section 2.2: OR is
 *   the operation the Index needs), or what adding the ranks' wire Indexes
 *   gives (see "Index modes"); counts its non-zeros U, derives the sketch
 *   layout (A, m_sub, m), the partition bounds and, per partition, the hash
 *   salt: the smallest of 0..15 under which no two non-zeros of the partition
 *   get the same three cells (such a pair could never be decoded; section
 *   2.2 and Table 1 call the compression lossless); writes shared->header,
 *   shared->bounds; clears shared->status; locates the bounds in every given
 *   rank's pair list (ranks[r].idx, ranks[r].cnt are read, the ranges written
 *   behind the counts in ranks[r].cnt).
 * PHASE_SKETCH: shared->sketch[c] = ((ranks[0].sketch[c] + ranks[1].sketch[c])
 *   + ...) in rank order, float32, for c < m (16-bit wire cells are widened
 *   first).
 * `ranks` is a host array of n_ranks structs (1 <= n_ranks <= config.n_ranks).
 */
int tagc_aggregate(const tagc_plan_t *plan, uint32_t phase,
                   const tagc_rank_buffers *ranks, uint32_t n_ranks,
                   const tagc_shared_buffers *shared, void *stream);

/*
 * Algorithm 1: peeling_decompress(index, count_sketch) (section 2.2).
 * Enumerates the non-zeros of the merged Index in ascending order into
 * idx_out[0..U), peels the summed sketch (shared->sketch is consumed) and
 * writes val_out[0..U); entries peeling cannot recover are counted in
 * shared->status and get 0 or, by the plan's decode_mode, an estimate (with
 * TAGC_DECODE_ESTIMATE there is no peeling and every entry is an estimate).  If dense_out (dev, n_c floats) is not NULL the summed
 * gradient is also written densely over the whole c-index space (zeros
 * elsewhere).  idx_out / val_out: dev, union_capacity entries.
 */
int tagc_decompress(const tagc_plan_t *plan, const tagc_shared_buffers *shared,
                    uint32_t *idx_out, float *val_out, float *dense_out,
                    void *stream);

/*
 * Algorithm 1's last two steps in one call: Reduce(count_sketch) and
 * peeling_decompress(index, count_sketch) (section 2.2), for a master that
 * holds the N ranks' sketches in its own memory (on one GPU: always; across
 * GPUs: peers that write their sketches into the master's buffers).  Equal to
 * tagc_aggregate(PHASE_SKETCH) followed by tagc_decompress -- every cell is
 * the same float32 sum ((ranks[0].sketch[c] + ranks[1].sketch[c]) + ...) in
 * rank order, up to the sign of a zero -- except that the summed sketch is
 * never written or read back: part of the decoder's waves add up the next
 * partition's cells in registers while the others peel the current one.
 * shared->sketch is not touched; tagc_aggregate(PHASE_INDEX) must have run.
 * ranks: host array of n_ranks structs, 1 <= n_ranks <= min(config.n_ranks,
 * 32).  float32 cells and partitions of the default size at most
 * (part_unknowns <= 8192, part_cells <= 12288): TAGC_EUNSUPPORTED otherwise.
 * Outputs and status as tagc_decompress.
 */
int tagc_reduce_decompress(const tagc_plan_t *plan, const tagc_rank_buffers *ranks,
                           uint32_t n_ranks, const tagc_shared_buffers *shared,
                           uint32_t *idx_out, float *val_out, float *dense_out,
                           void *stream);

/*
 * Optional per-kernel timing.  While enabled, every kernel the library
 * launches is bracketed by HIP events on the caller's stream.
 * tagc_profile_read synchronises those events (call it after the stream is
 * idle), returns up to `cap` entries (kernel name, total milliseconds, launch
 * count), clears the record, and returns the number of distinct kernels or a
 * negative error.  Names are static strings owned by the library.
 */
int tagc_profile_enable(int on);
int tagc_profile_read(const char **names, double *total_ms, uint64_t *launches,
                      uint32_t cap);

const char *tagc_strerror(int err);

#ifdef __cplusplus
}
#endif
#endif /* TAGC_H */
