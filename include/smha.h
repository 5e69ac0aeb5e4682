/*
 * smha -- masked multi-head attention for AMD MI355X (gfx950), C ABI.
 *
 *   O = softmax(scale * Q K^T  restricted to the unmasked keys of each query) V
 *
 * computed only over the unmasked entries of a static mask.  The library follows the
 * "unified MHA module" of the STOF paper (Sec. 4.2): a mask is analysed once into a
 * per-row column-index format and a two-level block format (block-compressed sparse rows
 * plus a bitmap per partially filled tile, Sec. 4.2.1), an analytical selector
 * (Sec. 4.2.3, Eq. 1) picks a row-wise or a block-wise kernel, and the forward call runs
 * one fused kernel that never touches empty tiles (Sec. 4.2.2, Algorithm 1).
 *
 * Conventions
 *   - A mask entry of 1 means "query i attends key j".  A query with no unmasked key
 *     produces an all-zero output row (the paper does not define this case).
 *   - Self-attention has Sq = Sk = S; a dense mask may also have fewer or more queries than
 *     keys (smha_plan_from_dense_rect: cross-attention, a chunk of queries against cached
 *     keys).  head_dim d is a multiple of 8 up to 256 (the kernels exist for 64, 128 and 256
 *     columns; a narrower head runs on the next of them, its missing columns read as zeros).  Q/K/V are IEEE binary16 or bfloat16.
 *   - All functions return a status code; nothing is printed, thrown or aborted.
 *     On error, output parameters are left untouched.
 *   - "host" / "device" is stated per pointer.  The library never frees or keeps
 *     Q/K/V/O; it owns everything reachable from a plan.
 */
#ifndef SMHA_H
#define SMHA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct smha_plan smha_plan_t; /* opaque; created by smha_plan_from_*, freed by smha_plan_destroy */

typedef enum {
    SMHA_OK = 0,
    SMHA_ERR_INVALID_ARG = 1, /* null pointer, negative size, unknown enum value            */
    SMHA_ERR_UNSUPPORTED = 2, /* head_dim / block size / dtype / alignment not supported    */
    SMHA_ERR_SHAPE = 3,       /* B/H do not match the plan's mask broadcast shape, S < 1    */
    SMHA_ERR_ALLOC = 4,       /* host or device allocation failed                           */
    SMHA_ERR_HIP = 5          /* no usable GPU, or a HIP runtime call failed                */
} smha_status_t;

typedef enum { SMHA_F16 = 0, SMHA_BF16 = 1, SMHA_F32 = 2 /* output only */ } smha_dtype_t;
typedef enum { SMHA_KERNEL_AUTO = 0, SMHA_KERNEL_ROW = 1, SMHA_KERNEL_BLOCK = 2 } smha_kernel_t;
typedef enum {
    SMHA_SELECTOR_CALIBRATED = 0, /* cost model fitted to MI355X measurements (default)       */
    SMHA_SELECTOR_PAPER_EQ1 = 1   /* the paper's formula verbatim (Sec. 4.2.3, Eq. 1)         */
} smha_selector_t;

/* Plan options.  Zero-initialise for defaults. */
typedef struct {
    int block;      /* tile edge of the exported block format: 16, 32 or 64; 0 = 64 (the paper's
                       OuterTile, Sec. 4.2.1)                                                  */
    int force;      /* smha_kernel_t; AUTO lets the selector decide                            */
    int selector;   /* smha_selector_t                                                         */
    int build_both; /* nonzero: keep both formats so either kernel can be forced at run time  */
    int device_id;  /* >= 0: upload index arrays to that GPU at plan time; -1: the current
                       device if there is one, otherwise stay host-only (forward then returns
                       SMHA_ERR_HIP); -2: host-only on purpose                                 */
    int head_dim;   /* hint for the calibrated selector (0 = 64)                               */
    int no_gather;  /* nonzero: the block kernel visits every non-empty 64x64 tile as it is; 0: tiles
                       with few used key columns are repacked into gathered tiles (block kernel
                       work lists only; the exported formats are never affected)               */
    int block_form; /* which form of the block-wise kernel runs where several exist: 0 = the library's choice
                       (at 128 columns form 3, unless nearly all tiles are full and the lists long: form 1;
                       at 256 columns form 3; at 64 columns form 1),
                       1 = four waves per workgroup, every wave forms scores, probabilities and output of
                       its 32 rows (one to four workgroups per compute unit); 2 = eight waves per workgroup,
                       score waves and value waves, one workgroup per compute unit (64 and 128 columns);
                       3 = eight waves of 16 rows per workgroup, two workgroups per compute unit at 128
                       columns, one at 256.  Plans with gathered tiles always run form 1, as does bfloat16
                       at 128 columns where form 2 is asked for.  For measurements and tests.             */
} smha_plan_opts_t;

/* Mask description: the atomic patterns of the paper (Sec. 2.1.2, Fig. 1) and their
 * compounds.  Composition:
 *     M = (WINDOW | GLOBAL | STRIDED | BLOCK_RANDOM | BIGBIRD   [all ones if none is set])
 *         & CAUSAL (if set) & PADDING (if set)
 * Random components use a counter-based generator: u = top 53 bits of
 * mix(mix(seed ^ mix(head)) ^ (block_row << 32 | block_col)) / 2^53 with mix = the
 * splitmix64 output function, head = 0 unless per_head. */
enum {
    SMHA_MASK_CAUSAL = 1,        /* keep j <= i                                                */
    SMHA_MASK_WINDOW = 2,        /* keep i - j <= window_left and j - i <= window_right        */
    SMHA_MASK_GLOBAL = 4,        /* keep rows i < n_global and columns j < n_global            */
    SMHA_MASK_STRIDED = 8,       /* keep j % stride == stride_phase                            */
    SMHA_MASK_BLOCK_RANDOM = 16, /* keep block (br, bc) iff u < keep_p, and every br == bc     */
    SMHA_MASK_BIGBIRD = 32,      /* per block row: n_window_blocks columns centred on br,
                                    the first n_global_blocks block rows and columns, and the
                                    n_random_blocks not-yet-kept columns of smallest (hash, bc) */
    SMHA_MASK_PADDING = 64       /* keep only i < valid_len[b] and j < valid_len[b]            */
};

typedef struct {
    uint32_t flags;
    int window_left, window_right;
    int n_global;
    int stride, stride_phase;
    int block; /* block edge of BLOCK_RANDOM / BIGBIRD (any positive size)                    */
    double keep_p;
    int n_window_blocks, n_global_blocks, n_random_blocks;
    uint64_t seed;
    int per_head;             /* random components differ per head: one mask per head          */
    const int32_t *valid_len; /* host, [B]; required with PADDING: one mask per batch entry    */
} smha_mask_desc_t;

typedef struct {
    int S, Bm, Hm;      /* queries per sequence; masks are [Bm][Hm][S][Sk], Bm in {1,B}, Hm in {1,H} */
    int block;          /* tile edge of the exported block format                               */
    int kernel;         /* SMHA_KERNEL_ROW or SMHA_KERNEL_BLOCK: what smha_forward will run     */
    int has_row_format, has_block_kernel_lists, on_device;
    int64_t nnz;        /* unmasked entries, summed over the Bm*Hm masks                         */
    int64_t n_valid, n_full, n_part; /* tiles of edge `block`, summed over masks                 */
    int64_t n_valid16;  /* non-empty 16x16 tiles, summed over masks (input of Eq. 1)             */
    int64_t n_tiles64;  /* non-empty 64x64 tiles the block kernel visits, summed over masks      */
    int64_t n_union;    /* K/V tile loads of the block kernel: union of the tile lists of the two
                           tile rows each 128-row workgroup covers, summed over masks             */
    int64_t n_items, n_split_rows; /* block-kernel work items / 128-row groups split along keys  */
    double eq1_threshold; /* Eq. 1 with valid16 averaged over masks; < 0 means row-wise          */
    double model_row_us, model_block_us; /* calibrated cost model, per (batch, head) pair         */
    int Sk;             /* keys per sequence (= S unless the plan came from smha_plan_from_dense_rect) */
    int64_t n_gathered; /* gathered tiles in the block kernel's lists (each replaces several sparse tiles) */
} smha_plan_info_t;

/* Arrays smha_plan_export can copy out (all host byte order, packed):
 *   ROW_PTR int32[S+1], COL_IDX int32[nnz]  -- per-row format, columns ascending in a row
 *   LOAD/FULL/PART_ROW_PTR int32[nbr+1], LOAD/FULL/PART_COL_IDX int32[...]  (Sec. 4.2.1;
 *     nbr = ceil(S/block); load = full U part, ascending inside a tile row)
 *   BLOCK_FLAGS uint8 per load entry: 1 = full (all block*block entries unmasked), 0 = part
 *   BITMAP uint64[n_part][block], part tiles in PART_COL_IDX order: word r = tile row r,
 *     bit c (LSB = 0) = tile column c; entries past S are 0, so a ragged tile is never full
 *   BITMAP_IT8 uint64[n_part][64] (block == 64 only): the paper's inner-tile layout, word
 *     ic*8+ir = 8x8 inner tile (ir, ic) (column-major over inner tiles), bit 8*r+c = entry (r,c)
 * The block kernel's own work lists (for inspection and tests; UNSUPPORTED if the plan has none):
 *   KERNEL_ITEMS int32[n_items of this mask][8]: {128-row group, first entry, end entry, workspace slot
 *     or -1, first gathered tile, gathered tiles, split group (index among this mask's split groups)
 *     or -1, 0}
 *   KERNEL_ITEMS_FINE: the same groups cut to at most 16 entries per item; smha_forward walks these
 *     instead when the call has too few items to fill the chip (few heads, long lists), so that the
 *     longest list does not set the launch's duration
 *   KERNEL_ENTRIES int32[n][4], all masks: {key tile, code for the group's first 64 rows, code for its
 *     second 64 rows, gathered tile + 1 or 0}; code -2 = nothing, -1 = every entry set, >= 0 = block
 *     of KERNEL_BITMAPS.  An ordinary entry covers keys 64*tile .. 64*tile+63; a gathered one the 64
 *     keys KERNEL_GATHER_KEYS[gathered tile][0..63] (keys >= Sk are padding)
 *   KERNEL_BITMAPS uint64[n][64]: word r = query row r of the 64, bit k = k-th key of the entry
 *   KERNEL_GATHER_KEYS int32[n][64]
 */
typedef enum {
    SMHA_EXPORT_ROW_PTR = 0,
    SMHA_EXPORT_COL_IDX = 1,
    SMHA_EXPORT_LOAD_ROW_PTR = 2,
    SMHA_EXPORT_LOAD_COL_IDX = 3,
    SMHA_EXPORT_BLOCK_FLAGS = 4,
    SMHA_EXPORT_BITMAP = 5,
    SMHA_EXPORT_FULL_ROW_PTR = 6,
    SMHA_EXPORT_FULL_COL_IDX = 7,
    SMHA_EXPORT_PART_ROW_PTR = 8,
    SMHA_EXPORT_PART_COL_IDX = 9,
    SMHA_EXPORT_BITMAP_IT8 = 10,
    SMHA_EXPORT_KERNEL_ITEMS = 11,
    SMHA_EXPORT_KERNEL_ENTRIES = 12,
    SMHA_EXPORT_KERNEL_BITMAPS = 13,
    SMHA_EXPORT_KERNEL_GATHER_KEYS = 14,
    SMHA_EXPORT_KERNEL_ITEMS_FINE = 15
} smha_export_t;

/* Mask analysis (Sec. 4.2.1) from a dense boolean mask.
 *   mask            uint8 [Bm][Hm][S][S], nonzero = attend; host pointer if mask_on_device
 *                   is 0, else a device pointer on the current device.  A device mask is
 *                   analysed by GPU kernels on the default stream: tile by tile (16 bytes per
 *                   64x64 tile and the bitmaps of partially filled tiles cross to the host) when
 *                   the plan needs no per-row lists and exports 64-wide tiles, else packed to bit
 *                   rows (1/8 of the bytes cross over) for the host analysis.  Either way the
 *                   plan equals the one built from the same mask in host memory, and the call
 *                   synchronises before returning
 *   opts            may be NULL (defaults)
 *   out             receives the plan
 * Errors: INVALID_ARG (null, Bm/Hm/S < 1), UNSUPPORTED (block), ALLOC, HIP. */
smha_status_t smha_plan_from_dense(const uint8_t *mask, int mask_on_device, int Bm, int Hm, int S,
                                   const smha_plan_opts_t *opts, smha_plan_t **out);

/* The same for a mask with Sq queries and Sk keys per sequence, uint8 [Bm][Hm][Sq][Sk] (the
 * per-row definition of attention does not need Sq = Sk; Sec. 2.1.1).  Row arrays then have Sq + 1
 * entries, tile rows cover queries and tile columns keys; for Eq. 1 the valid-tile ratio is taken
 * over the ceil(Sq/16) * ceil(Sk/16) tiles and n = ceil(Sk/16).  smha_forward takes Q and O with
 * Sq rows and K and V with Sk rows.  smha_plan_from_dense is the case Sq = Sk. */
smha_status_t smha_plan_from_dense_rect(const uint8_t *mask, int mask_on_device, int Bm, int Hm, int Sq, int Sk,
                                        const smha_plan_opts_t *opts, smha_plan_t **out);

/* Mask analysis from a pattern description; B and H fix how many distinct masks exist
 * (Bm = B with PADDING else 1; Hm = H with per_head and a random component, else 1). */
smha_status_t smha_plan_from_desc(const smha_mask_desc_t *desc, int B, int H, int S,
                                  const smha_plan_opts_t *opts, smha_plan_t **out);

smha_status_t smha_plan_info(const smha_plan_t *plan, smha_plan_info_t *out);

/* Copy one index array of mask `mask_index` (= bm*Hm + hm) to host memory.
 * *need receives the size in bytes; if cap < *need nothing is copied and the call still
 * returns SMHA_OK (query-then-copy).  host_dst may be NULL when cap is 0.
 * UNSUPPORTED if the plan does not hold that array (e.g. ROW_PTR of a block-only plan). */
smha_status_t smha_plan_export(const smha_plan_t *plan, int mask_index, smha_export_t which,
                               void *host_dst, size_t cap, size_t *need);

/* Fused masked attention (Sec. 4.2.2, Algorithm 1 for the block kernel; Sec. 4.1 for the
 * row-wise kernel).  Enqueues on `hip_stream` (a hipStream_t, NULL = default stream) and
 * returns without synchronising.
 *   Q               device, [B][H][S][d] of in_dtype, addressed through *_strides
 *   K, V            device, [B][H][Sk][d] of in_dtype (Sk = S for self-attention plans)
 *   O               device, [B][H][S][d] of out_dtype (same as in_dtype, or SMHA_F32)
 *   *_strides       host, {batch, head, seq} strides in elements, d is contiguous;
 *                   NULL = packed.  Pointers must be 16-byte aligned, strides multiples of
 *                   8 elements, the seq stride at least d, and one (batch, head) slice of
 *                   each tensor must span less than 2 GiB (UNSUPPORTED otherwise).
 *   scale           <= 0 selects 1/sqrt(d)
 *   kernel          AUTO = the plan's choice; ROW/BLOCK need that format in the plan
 * What the block kernel needs per call shape (B, H, d) beyond the plan's index arrays -- the work
 * order and the workspaces of split 128-row groups, see smha_plan_prepare -- is made by that
 * function or, if the shape was never prepared, by the first forward that uses it (that one call
 * allocates device memory and copies to it, so it must not be captured into a HIP graph; every later
 * call, and every call with a prepared shape, allocates, frees and synchronises nothing).  Nothing
 * made for a shape is freed or moved before smha_plan_destroy, so captured graphs and queued
 * launches stay valid whatever other shapes are used later.  Forwards on one plan may overlap on
 * different streams: successive calls with one shape take its 4 workspaces in turn, so up to 4 of
 * them may be in flight at once (a fifth would share the first one's workspace: serialise it
 * behind that call).
 * Errors: INVALID_ARG, UNSUPPORTED (d, dtype, alignment, missing format, more than 2^28
 * work items in one call), SHAPE, ALLOC, HIP. */
smha_status_t smha_forward(const smha_plan_t *plan, const void *Q, const void *K, const void *V,
                           void *O, int B, int H, int d, smha_dtype_t in_dtype,
                           smha_dtype_t out_dtype, const int64_t q_strides[3],
                           const int64_t k_strides[3], const int64_t v_strides[3],
                           const int64_t o_strides[3], float scale, smha_kernel_t kernel,
                           void *hip_stream);

/* smha_forward for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, same result, but the partial
 * results of split 128-row groups go to an array inside the library's own image (32 MiB per GPU,
 * held until the process ends) instead of a workspace of the plan, and nothing is ever allocated,
 * freed or synchronised.  The call shape must have been prepared (smha_plan_prepare, or an earlier
 * smha_forward with the same B, H, d): UNSUPPORTED otherwise, and also when the shape's workspace
 * (see smha_plan_prepare) exceeds the 32 MiB.  A small kernel clears the array's arrival counters
 * ahead of the attention kernel, on the same stream.  Every call on a GPU shares that GPU's one
 * array: calls that overlap in time on one GPU (two streams, two plans, two threads) race on it and
 * must be serialised by the caller; calls that follow each other on one stream are fine.  Plans that
 * split nothing, and the row-wise kernel, do not touch the array.
 * Errors: as smha_forward, plus UNSUPPORTED as described. */
smha_status_t smha_forward_static(const smha_plan_t *plan, const void *Q, const void *K, const void *V,
                                  void *O, int B, int H, int d, smha_dtype_t in_dtype,
                                  smha_dtype_t out_dtype, const int64_t q_strides[3],
                                  const int64_t k_strides[3], const int64_t v_strides[3],
                                  const int64_t o_strides[3], float scale, smha_kernel_t kernel,
                                  void *hip_stream);

/* Makes, once, everything smha_forward needs for calls with this batch size, head count and head
 * size on a plan that runs the block-wise kernel (Sec. 4.2.2): the work order (which workgroup
 * takes which work item, see smha_plan_work_order) and 4 workspaces that hold the partial results
 * of 128-row groups whose tile lists were split between workgroups (those are merged inside the
 * same launch by whichever part finishes last) -- B*H * (split parts per head) * (128 D + 1024)
 * floats each, D the kernel width for d (64, 128 or 256); plans that split nothing get none.
 * Allocates device memory and copies to it (blocking); call it outside stream capture, on the plan's device.  Calling it again for the
 * same shape does nothing; plans that run the row-wise kernel need nothing and return SMHA_OK.
 * Errors: INVALID_ARG, UNSUPPORTED (d, more than 2^28 work items), SHAPE, ALLOC, HIP. */
smha_status_t smha_plan_prepare(const smha_plan_t *plan, int B, int H, int d);

/* The block kernel's work order for B x H heads when workgroups_per_xcd workgroups are
 * resident on each of the chip's 8 XCDs (smha_forward uses 4 per compute unit at 64 columns,
 * 2 at 128, 1 at 256): the plan's work items (the workgroup tiling of Algorithm 1's outer loop)
 * differ in length, and each head's items go, longest first, to the workgroup with the
 * least work so far.  For inspection and tests; runs on the host.
 *   fine       0: the items of SMHA_EXPORT_KERNEL_ITEMS, 1: those of KERNEL_ITEMS_FINE
 *   host_dst   host, int32: 8 list starts (in pairs), 8 list lengths (in pairs), then the
 *              lists: (batch*head, index into that grain's items of all masks, masks in
 *              order) pairs.  XCD x serves the heads with batch*head mod 8 = x; the
 *              workgroup of rank r takes positions r, r + *per_xcd, ... of its XCD's list
 *              until the list ends or a pair with batch*head = -1 (no more work for this
 *              rank) comes up.
 *   cap, need  capacity of host_dst and the size needed, in int32 words (call with cap 0
 *              to learn the size); nothing is written if cap < *need
 *   per_xcd    workgroups per XCD actually used (<= workgroups_per_xcd); may be NULL
 * Errors: INVALID_ARG, SHAPE (B, H against the plan's masks), UNSUPPORTED (no block format). */
smha_status_t smha_plan_work_order(const smha_plan_t *plan, int B, int H, int workgroups_per_xcd,
                                   int fine, int32_t *host_dst, size_t cap, size_t *need,
                                   int *per_xcd);

void smha_plan_destroy(smha_plan_t *plan); /* NULL is allowed */

const char *smha_status_string(smha_status_t status);

/* Name and average duration bookkeeping is left to the caller; this returns the symbol
 * name of the kernel smha_forward would launch, for matching profiler output. */
const char *smha_kernel_name(const smha_plan_t *plan, int d, smha_dtype_t in_dtype,
                             smha_kernel_t kernel);

#ifdef __cplusplus
}
#endif
#endif /* SMHA_H */
