/*
 * dam.h -- C ABI of the DAM (Dynamic Attention Mask) hot path for AMD MI355X (gfx950).
 *
 * The operations, all enqueued on a caller-supplied HIP stream:
 *
 *   dam_mask_build            attention statistics captured at length L  ->  per-head sparse mask
 *                             (paper Sec. 4.2.2 - 4.2.4 and Sec. 4.3), emitted as an element bitmask
 *                             pooled by tile plus a compressed block index, and optionally as
 *                             per-row kept-key lists and a dense bitmask.
 *   dam_capture_accumulate    attention probabilities of a captured sequence summed into those
 *                             statistics (paper Sec. 4.2.1 - 4.2.2); dam_mask_build_from_qk fuses one
 *                             capture with the mask build.
 *   dam_sparse_attn_prefill   masked causal self-attention over the kept (query, key) entries only
 *                             (paper Sec. 3 and the last two equations of Sec. 4.3).
 *   dam_sparse_attn_decode    the same formula for one new query row per (sequence, head), reading
 *                             only the kept K/V rows.
 *   dam_kv_evict_plan, dam_kv_compact, dam_kv_remap_lists   drop the cached keys no future row of a
 *                             pattern mask attends and decode from the compacted cache (paper Sec. 2).
 *
 * Conventions shared by every entry point
 *   - Plain C. "device" pointers are HIP device addresses, "host" pointers are ordinary host memory.
 *     Parameter structs are host memory and are read before the call returns.
 *   - Ownership: every buffer (inputs, outputs, workspace) is allocated and freed by the caller.
 *     The library keeps no state between calls and allocates nothing (one stated exception:
 *     dam_sparse_attn_decode_grouped_static and its fixed scratch array).
 *   - Asynchrony: all device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream). No entry point synchronises the host. Device scalars written by a call
 *     (bmin, blk_total, kept_total) are valid once the caller has synchronised the stream.
 *   - Errors: the return value only (a dam_status). Argument errors are detected on the host
 *     before anything is launched; in that case no output is touched.
 *   - All indices are 0-based. Causality (key j <= query i) is part of every mask.
 *   - Masks belong to a (layer, head) pair, not to an input, so one mask serves every batch entry.
 */
#ifndef DAM_H
#define DAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DAM_OK = 0,
  DAM_ERR_INVALID_ARG = -1, /* null required pointer, non-positive size, hq % hkv != 0, bad ranges */
  DAM_ERR_UNSUPPORTED = -2, /* a head_dim / dtype / tile / lambda outside the built set          */
  DAM_ERR_WORKSPACE = -3,   /* ws_bytes smaller than the matching *_workspace() query             */
  /* -4 is not used: a capacity overflow cannot be known on the host without a synchronisation. It is
     reported through the device scalars blk_total / kept_total / col_total, and the offsets written
     never exceed the capacity (see dam_mask_out).                                                 */
  DAM_ERR_DEVICE = -5       /* a kernel launch failed                                              */
} dam_status;

typedef enum { DAM_F32 = 0, DAM_BF16 = 1 } dam_dtype;

/* dam_mask_params.transform: the method's Box-Cox, or one of the alternatives of App. B ("Feature
 * Amplification Transformation Methods"), with X = max(Abar, eps); the global minimum of the result is
 * subtracted before the threshold in every case.
 *   raw sum A; average Abar; log ln X; Yeo-Johnson ((X+1)^lambda - 1)/lambda, ln(X+1) at lambda 0;
 *   z-score (X - mean X)/(std X + eps) and min-max (X - min X)/((max X - min X) + eps), statistics over
 *   every stored entry of every map of the call; square root; arcsinh.
 * raw sum, average, min-max and square root are exact fp32 sequences like the Box-Cox path; log,
 * Yeo-Johnson, arcsinh (library functions) and z-score (fp64 sums in no fixed order) can decide
 * entries within rounding of the threshold differently from another implementation. Any lambda is
 * accepted for Yeo-Johnson. FROM_ATTN_MAP only; dam_mask_build_from_qk takes Box-Cox only. */
typedef enum {
  DAM_T_BOXCOX = 0, DAM_T_RAW_SUM = 1, DAM_T_AVERAGE = 2, DAM_T_LOG = 3, DAM_T_YEO_JOHNSON = 4,
  DAM_T_ZSCORE = 5, DAM_T_MINMAX = 6, DAM_T_SQRT = 7, DAM_T_ARCSINH = 8
} dam_transform;

/* dam_mask_params.flags */
typedef enum {
  DAM_MASK_SKIP_FULL_TILE_BITS = 1, /* do not write tile_bits of full tiles (blk_kind bit 0): the attention
                                      kernels never read them, and at long sequences they are a large part
                                      of the bytes written. Their slots in the pool stay reserved and keep
                                      whatever they held.                                                  */
  DAM_MASK_GATHER_COLUMNS = 2,      /* list the matched columns in tiles of their own. The mask is the same;
                                      in every query tile that lies wholly in the pattern region (first row
                                      >= pcl) its entries are split into
                                        a diagonal part: key j <= i with i - j a matched diagonal, listed in
                                          the ordinary tiles (tile index < nKt = ceil(S / tile_n)), and
                                        a column part: matched column c <= i with i - c NOT a matched
                                          diagonal, listed in "gathered" tiles with index nKt + v: key slot
                                          s of gathered tile v stands for column gather_idx[h][v tile_n + s].
                                      A vertical stripe then costs its share of one dense tile per query
                                      tile instead of a tile of its own. Query tiles that start inside the
                                      true-mask block are listed as without the flag. Requires the outputs
                                      gather_idx and gather_cnt.                                          */
  DAM_MASK_GROUP_LISTS = 4,         /* kept lists for grouped-query decoding: one list per group of
                                      `group` consecutive maps (the query heads of one KV head) instead of
                                      one per map, so that a decode step reads every cached row once for
                                      the whole group. The list of a group holds each key kept by any of
                                      its maps once, in G + 1 runs, each ascending: the keys kept by two or
                                      more of the maps, then those kept by map 0 of the group alone, by map
                                      1 alone, ... kept_member[e] has bit x set iff map x of the group
                                      keeps key kept_idx[e]. One row only (row_end = row_begin + 1);
                                      n_maps a multiple of group, 1 <= group <= 8; requires kept_member
                                      when kept_idx is given.                                              */
  DAM_MASK_PATTERN_PLAN = 8         /* with DAM_MASK_GROUP_LISTS: the lists do not depend on the position and serve
                                      every row of the pattern region (row p >= pcl keeps key j <= p iff p - j is a
                                      matched diagonal or j is a matched column), so a decode loop builds them once
                                      per mask instead of once per step. The list of a group holds first every
                                      diagonal offset r matched by some map of the group, then every such column
                                      c < min(P, seq), each part in G + 1 runs (patterns of two or more maps; of map
                                      0 alone; of map 1 alone; ...), each run ascending in the key it stands for
                                      (diagonals by descending offset). kept_idx[e] is -1 - r for a diagonal (key
                                      p - r at position p) and c for a column; kept_member[e] names the maps that
                                      have the pattern. plan_table [n_maps / group][P] u8 (required): the member
                                      bits of every diagonal offset; at position p a column entry c serves the maps
                                      in kept_member & ~plan_table[group][p - c], the others meet key c through
                                      their diagonal already. row_begin / row_end are ignored. Consumed by
                                      dam_sparse_attn_decode_patterns.                                       */
} dam_mask_flags;

typedef enum {
  DAM_FROM_ATTN_MAP = 0, /* derive the true mask and the matched patterns from A (and C)          */
  DAM_FROM_PATTERNS = 1  /* matched patterns (and optionally a true mask) are supplied            */
} dam_mask_mode;

/* ------------------------------------------------------------------------------------------------
 * dam_mask_build
 *
 * Sec. 4.2.2:  Abar = A / (C + eps);  X = max(Abar, eps);  B = (X^lambda - 1) / lambda;
 *              Bstar = B - min over every map and entry of the call (or bmin_override).
 * Sec. 4.2.3:  true mask  m[i][j] = (Bstar[i][j] >= tau)  and  j <= i,   an L x L matrix per map.
 * Sec. 4.2.4:  match score of the diagonal pattern r (entries j = i - r) and of the vertical pattern c
 *              (entries j = c, i >= c):  gamma = (kept entries on the pattern) / (entries of the
 *              pattern);  a pattern is matched when gamma >= mu.
 * Sec. 4.3:    mask of an S x S problem.  S <= L: the top-left S x S crop of m.   S > L: m inside the
 *              top-left L x L block; elsewhere entry (i, j), j <= i, is kept iff (i - j) is a matched
 *              diagonal or j is a matched column.
 *
 * The arithmetic of the first three steps is a fixed fp32 sequence, each operation rounded to
 * nearest-even and never contracted: abar = a / (c + eps); x = max(abar, eps);
 * lambda = 0.5: b = (sqrt(x) - 1) / 0.5;  lambda = 1: b = x - 1;  keep = (b - bmin) >= tau;
 * gamma = (float)count / (float)length; matched = gamma >= mu.  Other lambda: DAM_ERR_UNSUPPORTED.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t mode;      /* dam_mask_mode                                                              */
  int32_t n_maps;    /* H: number of (layer, head) maps handled by this call                        */
  int32_t pcl;       /* L: pattern capture length (FROM_ATTN_MAP: below 131072, else
                        DAM_ERR_UNSUPPORTED). FROM_PATTERNS: side of the supplied true mask, or
                        0 when there is none (then the pattern rule applies everywhere)             */
  int32_t seq;       /* S: length of the problem the mask is built for                              */
  int32_t tile_m;    /* block-index tile, query rows;  multiple of 64, at most 256                  */
  int32_t tile_n;    /* block-index tile, key columns; multiple of 64, at most 256                  */
  int32_t row_begin; /* kept lists are emitted for rows [row_begin, row_end) of the S x S mask      */
  int32_t row_end;   /*   (0 <= row_begin <= row_end <= S); ignored when kept_ptr is NULL           */
  float lambda;      /* Box-Cox exponent: 0.5 (the paper's) or 1                                    */
  float eps;         /* epsilon of the mean and of the clamp, > 0 (paper: 1e-8)                     */
  float tau;         /* true-mask threshold (paper: 0.3)                                            */
  float mu;          /* pattern-match threshold (paper: 0.8)                                        */
  float bmin_override; /* NaN: use the minimum over this call's maps; otherwise this value is bmin  */
  int32_t flags;     /* bit set of dam_mask_flags                                                   */
  int32_t transform; /* dam_transform: the step between the mean map and the threshold (0: Box-Cox)  */
  int32_t group;     /* DAM_MASK_GROUP_LISTS: maps per group (query heads per KV head); else ignored */
} dam_mask_params;

/* Outputs of dam_mask_build. Every pointer is a device pointer owned by the caller; any of them may
 * be NULL when that output is not wanted (exceptions are stated).
 *
 * Capacity: when the listed tiles (the kept keys) outnumber blk_capacity (kept_capacity), nothing is
 * written at or past the capacity, blk_total (kept_total) still holds the number required, and every
 * offset written to blk_row_ptr (kept_ptr) is cut to the capacity: the index then lists exactly the
 * first `capacity` tiles (keys), in order, and is safe to hand to the attention kernels (their result
 * is that of the truncated mask). In a sizing call (blk_col, blk_kind and tile_bits all NULL; kept_idx
 * NULL) the offsets are the true ones.
 *
 *   true_bits  [H][L][ceil(L/64)] u64   bit (j % 64) of word j / 64 of row i is m[i][j].
 *                                       FROM_ATTN_MAP: written, and required (the later steps of the
 *                                       same call read it back). FROM_PATTERNS: an input, read when
 *                                       pcl > 0, never written.
 *   diag_cnt, vert_cnt [H][L] i32       kept entries on each diagonal / column of the true mask
 *                                       (FROM_ATTN_MAP only).
 *   diag_flag, vert_flag [H][L] u8      1 = matched (FROM_ATTN_MAP only; when NULL the flags live in
 *                                       the workspace). In FROM_PATTERNS mode nothing is written here:
 *                                       the matched sets are the inputs diag_in / vert_in, [H][S].
 *   bmin       [1] f32                  the minimum used by the threshold.
 *   blk_row_ptr [H][nQt + 1] i32        CSR offsets into blk_col; offsets are global over all maps
 *                                       (blk_row_ptr[h][0] == blk_row_ptr[h-1][nQt]),
 *                                       nQt = ceil(S / tile_m). Required for any block output.
 *   blk_col    [blk_capacity] i32       key-tile index of each listed tile, ascending per query tile.
 *                                       A tile is listed iff it holds at least one kept entry.
 *   blk_kind   [blk_capacity] u8        bit 0: every entry of the tile is kept (the tile then lies
 *                                       strictly below the diagonal and inside S). Bits 1..4: key
 *                                       quarter q of the tile, columns [q tile_n/4, (q+1) tile_n/4),
 *                                       holds a kept entry (bit 1 + q); the attention kernel skips
 *                                       empty quarters.
 *   tile_bits  [blk_capacity][tile_m][tile_n / 64] u64   element bits of listed tile t at index t
 *                                       (also for full tiles: all ones, unless the flag
 *                                       DAM_MASK_SKIP_FULL_TILE_BITS is set); bits beyond S are 0.
 *   blk_total  [1] i64                  number of listed tiles, valid even when it exceeds
 *                                       blk_capacity (nothing is written past the capacity). Call
 *                                       with blk_col == NULL to size the buffers.
 *   dense_bits [H][S][ceil(S/64)] u64   the whole mask; only sensible for small S.
 *   kept_ptr   [H * (row_end - row_begin) + 1] i32   CSR offsets into kept_idx, map-major.
 *   kept_idx   [kept_capacity] i32      kept keys of each emitted row, ascending, no duplicates.
 *   kept_total [1] i64                  number of kept keys over the emitted rows (as blk_total).
 *   With DAM_MASK_GROUP_LISTS: kept_ptr [H / group + 1], one list per group; kept_member
 *   [kept_capacity] u8 beside kept_idx.
 */
typedef struct {
  uint64_t *true_bits;
  int32_t *diag_cnt, *vert_cnt;
  uint8_t *diag_flag, *vert_flag;
  float *bmin;
  int32_t *blk_row_ptr, *blk_col;
  uint8_t *blk_kind;
  uint64_t *tile_bits;
  int64_t blk_capacity;
  int64_t *blk_total;
  uint64_t *dense_bits;
  int32_t *kept_ptr, *kept_idx;
  int64_t kept_capacity;
  int64_t *kept_total;
  int32_t *gather_idx; /* [H][dam_gather_stride(params)] i32: DAM_MASK_GATHER_COLUMNS, the matched columns
                          below S of each map, ascending, then -1 up to the stride                        */
  int32_t *gather_cnt; /* [H] i32: how many                                                                */
  uint8_t *kept_member; /* [kept_capacity] u8: DAM_MASK_GROUP_LISTS, which maps of the group keep each entry */
  uint8_t *plan_table;  /* [H / group][P] u8: DAM_MASK_PATTERN_PLAN, member bits of every diagonal offset       */
} dam_mask_out;

/* Row length of gather_idx: min(P, S) rounded up to a multiple of tile_n, P the length of the pattern
 * flags (pcl from a map, S when patterns are given). 0 on invalid parameters. */
int32_t dam_gather_stride(const dam_mask_params *params);

/* Bytes of device workspace dam_mask_build needs for these parameters (0 on invalid parameters). */
size_t dam_mask_build_workspace(const dam_mask_params *params);

/* params     host.
 * attn_sum   device, f32 [H][L][L] row-major: A, attention summed over the captured batches.
 *            FROM_ATTN_MAP only (else NULL).
 * attn_cnt   device, f32 [H][L][L]: C, how often each pair was computed; or NULL, meaning one
 *            causal capture: C = 1 for j <= i and, for j > i, C = 0 and A is taken as 0 without
 *            being read.
 * diag_in, vert_in   device, u8 [H][S]: matched diagonal offsets / columns. FROM_PATTERNS only.
 * out        host struct of device pointers, see above.
 * ws         device workspace of at least dam_mask_build_workspace(params) bytes, 256-byte aligned.
 * Returns DAM_OK or a negative dam_status; on DAM_ERR_INVALID_ARG / UNSUPPORTED / WORKSPACE nothing
 * was launched. */
int dam_mask_build(const dam_mask_params *params, const float *attn_sum, const float *attn_cnt,
                   const uint8_t *diag_in, const uint8_t *vert_in, const dam_mask_out *out,
                   void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * dam_capture_accumulate, dam_mask_build_from_qk  (the step before the mask rule)
 *
 * Sec. 4.2.1 / 4.2.2: a sequence truncated to the pattern capture length is run with full causal
 * attention and its attention probabilities are summed into the statistics,
 *     A[h][i][j] += softmax_j(q_i . k_j * scale),   C[h][i][j] += 1      for j <= i < len,
 * over as many sequences as the caller captures (one call each). Query head h reads KV head
 * h / (hq / hkv). bf16 inputs use the matrix cores (head_dim 128) with fp32 accumulation, the
 * softmax is evaluated in fp32; the sums are fp32.
 *
 * dam_mask_build_from_qk is dam_mask_build (DAM_FROM_ATTN_MAP, attn_cnt == NULL) for ONE captured
 * sequence of exactly pcl tokens, fused with its capture: the probabilities are compared with the
 * threshold as they are produced and the map A is never written. Because the probabilities are
 * fp32 results of a different operation order than a stored map would have, true-mask bits of
 * entries whose probability lies within rounding distance of the threshold may differ from a build
 * that goes through a stored map; everything after the true mask is the same computation on
 * those bits.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t hq, hkv;
  int32_t len;          /* tokens of the captured sequence, 1 <= len <= pcl                        */
  int32_t pcl;          /* L: side of the statistics matrices                                      */
  int32_t head_dim;     /* 128 for the matrix-core path; any multiple of 8 up to 256 otherwise     */
  int32_t dtype;        /* dam_dtype of q and k                                                    */
  float scale;          /* logit scale; 0 means 1 / sqrt(head_dim)                                 */
  int64_t q_stride[2];  /* element strides of the head and position index; head_dim contiguous,    */
  int64_t k_stride[2];  /*   rows 16-byte aligned                                                  */
} dam_capture_params;

size_t dam_capture_workspace(const dam_capture_params *params);

/* q         device [hq][len][head_dim], k device [hkv][len][head_dim] by the strides above.
 * attn_sum  device f32 [hq][pcl][pcl], read and written (the caller zeroes it before the first
 *           capture). attn_cnt the same for the counts, or NULL.
 * ws        device workspace of at least dam_capture_workspace(params) bytes.
 * pcl up to 8192 and a position stride of k below 2^24 elements (DAM_ERR_UNSUPPORTED beyond). Errors as for
 * the other entry points. */
int dam_capture_accumulate(const dam_capture_params *params, const void *q, const void *k,
                           float *attn_sum, float *attn_cnt, void *ws, size_t ws_bytes, void *stream);

size_t dam_mask_build_from_qk_workspace(const dam_mask_params *params, const dam_capture_params *capture);

/* params    as for dam_mask_build; mode must be DAM_FROM_ATTN_MAP, n_maps == capture->hq,
 *           pcl == capture->pcl == capture->len (2 <= pcl <= 8192).
 * q, k      as above. out, ws, stream as for dam_mask_build (out->true_bits is required and written). */
int dam_mask_build_from_qk(const dam_mask_params *params, const dam_capture_params *capture, const void *q,
                           const void *k, const dam_mask_out *out, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * dam_sparse_attn_prefill
 *
 * Sec. 3 / Sec. 4.3: for every batch entry b, query head h and row i,
 *     O[i] = sum_{j in K_i} softmax_j(q_i . k_j * scale) v_j,   K_i = kept keys of row i of head h's
 * mask (masked entries are -inf before the softmax). A row without kept keys gives O[i] = 0 and
 * lse[i] = -inf. Query head h reads KV head h / (hq / hkv).
 * dtype DAM_BF16: bf16 in, fp32 accumulation on the matrix cores, bf16 out (round to nearest even);
 *                 head_dim 128, tiles 128 x 128; the rows of one K or V head must span less than
 *                 4 GiB (seq * stride[2] * 2 bytes), otherwise DAM_ERR_UNSUPPORTED. The softmax weights
 *                 are rounded to bf16 for the second product (see also DAM_ATTN_RUNNING_REFERENCE).
 * dtype DAM_F32:  fp32 throughout; head_dim 64 or 128, tiles of 64 or 128 in either direction.
 * A block index built with DAM_MASK_GATHER_COLUMNS is taken as it is: a tile index >= ceil(seq / tile_n)
 * names a gathered tile whose key slots are the columns in gather_idx (the bf16 kernel first copies
 * those K / V rows of every head into the workspace, so that such a tile is loaded like any other).
 * ---------------------------------------------------------------------------------------------- */
/* dam_attn_params.flags */
typedef enum {
  DAM_ATTN_RUNNING_REFERENCE = 1 /* bf16 kernel: evaluate every row with the running-maximum softmax. Without the
                                    flag the kernel first evaluates exp2(logit * log2 e) with no reference at all
                                    (two instructions per weight; exact while the weights fit fp32 / bf16, which
                                    share their 8 exponent bits), checks every row's sum of weights, and repeats
                                    the query tiles in which a sum left [2^-100, 2^100] with the running maximum.
                                    The results of that second pass are the flag's. Set it for inputs whose
                                    scaled logits are known to lie beyond about +-60: it saves the first pass. */
} dam_attn_flags;

typedef struct {
  int32_t batch, hq, hkv, seq, head_dim;
  int32_t dtype;        /* dam_dtype of q, k, v and out                                           */
  float scale;          /* logit scale; 0 means 1 / sqrt(head_dim)                                */
  int64_t q_stride[3];  /* element strides of the batch, head and sequence index; head_dim is     */
  int64_t k_stride[3];  /*   contiguous (stride 1). Rows must be 16-byte aligned.                 */
  int64_t v_stride[3];
  int64_t o_stride[3];
  int32_t tile_m, tile_n; /* the tile the block index was built with                              */
  int32_t gather_rows;    /* block index with gathered column tiles: an upper bound, a multiple of
                             tile_n, of gather_cnt[h] rounded up to tile_n over all heads (the rows of
                             the gathered K / V copies kept in the workspace); 0 otherwise           */
  int32_t flags;          /* bit set of dam_attn_flags                                            */
} dam_attn_params;

/* The block-index outputs of dam_mask_build for the hq query heads (device pointers). Device data
 * that the host cannot check: a blk_col entry outside the index's tile range is read as the nearest
 * tile inside it (the output is then meaningless, no address leaves K, V or the gathered copies);
 * blk_row_ptr must be a valid CSR offset array into buffers of at least that many tiles. */
typedef struct {
  const int32_t *blk_row_ptr; /* [hq][nQt + 1]                                                     */
  const int32_t *blk_col;
  const uint8_t *blk_kind;
  const uint64_t *tile_bits;
  const int32_t *gather_idx;  /* [hq][gather_stride], NULL unless built with DAM_MASK_GATHER_COLUMNS */
  const int32_t *gather_cnt;  /* [hq]                                                              */
  int32_t gather_stride;
} dam_mask_view;

size_t dam_sparse_attn_prefill_workspace(const dam_attn_params *params);

/* q, k, v, out  device, laid out by the strides above ([batch][heads][seq][head_dim] when dense).
 * lse           device f32 [batch][hq][seq] (natural-log sum-exp of the kept logits) or NULL.
 * ws            device workspace (may be NULL when the query returns 0). */
int dam_sparse_attn_prefill(const dam_attn_params *params, const void *q, const void *k,
                            const void *v, const dam_mask_view *mask, void *out, float *lse, void *ws,
                            size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * dam_sparse_attn_decode
 *
 * The formula above for one query row per (sequence b, query head h): the row attends the keys
 * listed in kept_idx[kept_ptr[b*hq+h] .. kept_ptr[b*hq+h+1]), positions in that sequence's cache,
 * ascending and without duplicates (row p of the head's mask, Sec. 4.3). An empty list gives
 * O = 0, lse = -inf. bf16 (fp32 accumulation) or fp32; head_dim 64 or 128.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t batch, hq, hkv;
  int32_t kv_capacity;   /* rows allocated per (sequence, KV head) in the caches                   */
  int32_t head_dim;
  int32_t dtype;
  float scale;           /* 0 means 1 / sqrt(head_dim)                                            */
  int64_t q_stride[2];   /* element strides of batch and head; head_dim contiguous                */
  int64_t kv_stride[3];  /* element strides of batch, KV head and position, for both caches       */
  int64_t o_stride[2];
  int32_t shared_lists;  /* 0: one kept list per (sequence, head), kept_ptr has batch*hq + 1 entries;
                            1: one list per head, used by every sequence of the batch (all of them
                            sit at the same position: the mask belongs to the head, not to the input),
                            kept_ptr has hq + 1 entries                                             */
} dam_decode_params;

/* max_kept: upper bound of the kept keys of one (sequence, head) list. */
size_t dam_sparse_attn_decode_workspace(const dam_decode_params *params, int64_t max_kept);

/* q, out      device [batch][hq][head_dim] by the strides above.
 * kcache, vcache  device [batch][hkv][kv_capacity][head_dim] by kv_stride.
 * kept_ptr    device i32 [batch*hq + 1] ([hq + 1] with shared_lists); kept_idx device i32.
 * max_kept    the bound given to the workspace query (the library does not read kept_ptr on the
 *             host); every list must be no longer than it and every index < kv_capacity. The lists
 *             are device data that the host cannot check: an index outside [0, kv_capacity) is
 *             read as the nearest cache row (the output is then meaningless, no address leaves the
 *             cache); kept_ptr itself must be a valid CSR offset array.
 * lse         device f32 [batch][hq] or NULL. */
int dam_sparse_attn_decode(const dam_decode_params *params, const void *q, const void *kcache,
                           const void *vcache, const int32_t *kept_ptr, const int32_t *kept_idx,
                           int64_t max_kept, void *out, float *lse, void *ws, size_t ws_bytes,
                           void *stream);

/* dam_sparse_attn_decode for all query heads of a KV head at once (grouped-query attention: hq / hkv
 * query heads share the K and V rows of one KV head). The lists are those of dam_mask_build with
 * DAM_MASK_GROUP_LISTS and group = hq / hkv (<= 8): one per (sequence, KV head), or one per KV head with
 * shared_lists, holding every key that some head of the group keeps once, and kept_member[e] naming the
 * heads that keep it (bit x: query head hkv_index * group + x). Each listed row is read once and enters
 * the softmax state of exactly the heads named; the results equal those of dam_sparse_attn_decode on
 * the per-head lists up to the order of the fp32 sums, except for bf16 with head_dim 128, where the
 * products run on the matrix cores with the softmax weights rounded to bf16, as in the prefill: there
 * the two agree within the bf16 output tolerance (2e-2 max-abs), not to the last bit.
 * kept_ptr  device i32 [batch*hkv + 1] ([hkv + 1] with shared_lists); kept_idx i32 and kept_member u8
 *           device arrays of the same length. Entries of one list may come in any order, without
 *           duplicates; runs of entries with equal kept_member cost no arithmetic for the other heads.
 * max_kept  upper bound of the length of one list. Everything else as dam_sparse_attn_decode. */
size_t dam_sparse_attn_decode_grouped_workspace(const dam_decode_params *params, int64_t max_kept);
int dam_sparse_attn_decode_grouped(const dam_decode_params *params, const void *q, const void *kcache,
                                   const void *vcache, const int32_t *kept_ptr, const int32_t *kept_idx,
                                   const uint8_t *kept_member, int64_t max_kept, void *out, float *lse,
                                   void *ws, size_t ws_bytes, void *stream);

/* dam_sparse_attn_decode_grouped from a position-independent plan (dam_mask_build with DAM_MASK_GROUP_LISTS |
 * DAM_MASK_PATTERN_PLAN and group = hq / hkv): the row at position `pos` of every head's pattern mask (Sec. 4.3:
 * key j <= pos is kept iff pos - j is a matched diagonal or j is a matched column), evaluated without building a
 * list for that row. Every sequence of the batch sits at position pos (the query is the token at index pos, keys
 * 0 .. pos are cached); the plan belongs to the heads and serves the whole batch and every position of the
 * pattern region (pos >= the capture length of the masks; masks given as patterns: any pos).
 * plan_ptr [hkv + 1] i32, plan_val i32, plan_member u8: the kept_ptr / kept_idx / kept_member of that build;
 * plan_table u8 [hkv][n_flags]: its plan_table; n_flags: the length P of the pattern flags.
 * max_entries: upper bound of the length of one list of the plan. bf16, head_dim 128, hq / hkv <= 8 (otherwise
 * DAM_ERR_UNSUPPORTED). Workspace: dam_sparse_attn_decode_grouped_workspace with shared_lists = 1 and
 * max_kept = max_entries. Everything else as dam_sparse_attn_decode_grouped; the results are those of the
 * list form on the lists of row pos, up to the order of the fp32 sums. */
int dam_sparse_attn_decode_patterns(const dam_decode_params *params, const void *q, const void *kcache,
                                    const void *vcache, const int32_t *plan_ptr, const int32_t *plan_val,
                                    const uint8_t *plan_member, const uint8_t *plan_table, int32_t n_flags,
                                    int32_t pos, int64_t max_entries, void *out, float *lse, void *ws,
                                    size_t ws_bytes, void *stream);

/* dam_sparse_attn_decode_grouped for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation. The same kernels, with the
 * partial results of the list splits kept in a fixed array of DAM_DECODE_STATIC_SCRATCH_BYTES bytes of
 * device memory that belongs to the library (every GPU the library runs on holds its own copy until the
 * process ends). The call allocates nothing and synchronises nothing; inputs and outputs are the
 * caller's as before. A call whose dam_sparse_attn_decode_grouped_workspace() exceeds the array returns
 * DAM_ERR_WORKSPACE and launches nothing. All calls on one GPU share that GPU's array: calls that may
 * overlap there (different streams, several threads) race on it; calls on one stream do not. The array keeps
 * the last call's contents; nothing in it has to start at zero (every split writes its partial result
 * before the merge pass reads it). The first call made with a device current looks up the array's address on
 * that device and keeps it: the only state the library holds.
 * dam_sparse_attn_decode_grouped_static_limit() returns DAM_DECODE_STATIC_SCRATCH_BYTES. */
#define DAM_DECODE_STATIC_SCRATCH_BYTES (8u << 20)
size_t dam_sparse_attn_decode_grouped_static_limit(void);
int dam_sparse_attn_decode_grouped_static(const dam_decode_params *params, const void *q, const void *kcache,
                                          const void *vcache, const int32_t *kept_ptr, const int32_t *kept_idx,
                                          const uint8_t *kept_member, int64_t max_kept, void *out, float *lse,
                                          void *stream);

/* ------------------------------------------------------------------------------------------------
 * dam_kv_evict_plan, dam_kv_compact, dam_kv_remap_lists: KV-cache eviction for decode
 *
 * Sec. 2 (local attention patterns allow evicting the KV cache beyond the attention span) applied to
 * the mask of Sec. 4.3: in the pattern region row i keeps key j iff i - j is a matched diagonal or j is
 * a matched column. For the query heads of KV head g, a cached key j <= pos is still attended by some
 * row i >= pos iff j is a matched column of one of them, or j >= pos - r_max(g) (r_max: their largest
 * matched diagonal). Everything else can be dropped. The compacted cache of (sequence, g) holds
 *     rows [0, n_col(g))                 the live columns, ascending,
 *     rows [n_col(g), n_col(g) + W(g))   a ring, W = r_max + 1: key j at row n_col + j mod W,
 * so no row moves while the position advances: the caller writes the K / V row of a new key j to row
 * n_col + j mod W (it overwrites the key that has just left the window). Matched columns that first
 * become <= pos later change n_col: plan and compact again then (stripe columns lie below the capture
 * length, so this does not happen once pos has passed it).
 * Valid for rows of the pattern region only (pos >= pcl; masks given as patterns: always).
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t batch, hq, hkv;
  int32_t n_flags;            /* P: length of each flag array                                      */
  int32_t pos;                /* position of the newest cached key                                 */
  int32_t head_dim, dtype;    /* of the caches (dam_compact only); a row must be a multiple of 16 B */
  int32_t kv_capacity;        /* rows per (sequence, KV head) of the full caches                   */
  int32_t compact_capacity;   /* rows per (sequence, KV head) of the compacted caches              */
  int64_t kv_stride[3];       /* element strides of batch, KV head, position (full caches)         */
  int64_t compact_stride[3];  /* the same for the compacted caches                                 */
} dam_evict_params;

size_t dam_kv_evict_workspace(const dam_evict_params *params);

/* diag_flag, vert_flag  device u8 [hq][n_flags]: matched diagonals / columns per query head.
 * window    device i32 [hkv]: W(g) (0 when the group has no matched diagonal).
 * col_ptr   device i32 [hkv + 1], cols device i32 [col_capacity]: live columns per KV head, ascending.
 * rows      device i32 [hkv] or NULL: n_col(g) + W(g), the rows the compacted cache of g needs.
 * col_total device i64 [1]: number of live columns over all KV heads, valid even when it exceeds
 *           col_capacity (nothing is written past it); call with cols == NULL to size. */
int dam_kv_evict_plan(const dam_evict_params *params, const uint8_t *diag_flag, const uint8_t *vert_flag,
                      int32_t *window, int32_t *col_ptr, int32_t *cols, int64_t col_capacity, int32_t *rows,
                      int64_t *col_total, void *ws, size_t ws_bytes, void *stream);

/* Gathers the live rows of the full caches [batch][hkv][kv_capacity][head_dim] into the compacted
 * ones [batch][hkv][compact_capacity][head_dim] (device pointers, strides in params). Ring rows whose
 * key does not exist yet (pos + 1 < W) are left untouched. */
int dam_kv_compact(const dam_evict_params *params, const int32_t *window, const int32_t *col_ptr,
                   const int32_t *cols, const void *kcache, const void *vcache, void *kcompact, void *vcompact,
                   void *stream);

/* kept_slot[e] = row of key kept_idx[e] in its KV head's compacted cache, for the lists of
 * dam_sparse_attn_decode (kept_ptr device i32 [batch*hq + 1]); the order of a list is kept, so decode
 * from the compacted cache adds the same terms in the same order. For the merged lists of
 * dam_sparse_attn_decode_grouped (one per (sequence, KV head), kept_ptr [batch*hkv + 1]) pass params whose hq
 * is set to hkv: a list then belongs to the KV head of its index. With lists shared by the batch, batch = 1. */
int dam_kv_remap_lists(const dam_evict_params *params, const int32_t *window, const int32_t *col_ptr,
                       const int32_t *cols, const int32_t *kept_ptr, const int32_t *kept_idx,
                       int32_t *kept_slot, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Measurement helpers (no passage of the paper: they measure the chip's own ceilings, printed by the
 * benchmark next to the published peaks its roofline fractions divide by).
 *
 * dam_probe_mfma: `workgroups` workgroups of four waves, each wave issuing iters * 16
 *   v_mfma_f32_32x32x16_bf16 (32768 flop each) into four independent accumulators and nothing else.
 *   operands: device, 8 KiB of bf16 values (the A and B fragments); sink: device, one float (never
 *   written in practice). Flop launched: workgroups * 4 * iters * 16 * 32768.
 * dam_probe_stream_read: reads `bytes` (a multiple of 32 KiB is read completely) from src with 16-byte
 *   loads and discards them. src device, 16-byte aligned; sink device, one word.
 * Both only enqueue on `stream`; the caller times them. */
int dam_probe_mfma(const void *operands, float *sink, int32_t workgroups, int32_t iters, void *stream);
int dam_probe_stream_read(const void *src, size_t bytes, uint32_t *sink, int32_t workgroups, void *stream);

/* Library version, for the loader's sanity check. */
int dam_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DAM_H */
