/*
 * compact_attn.h -- C ABI of the Compact Attention block-sparse forward for MI355X (gfx950).
 *
 * The library computes softmax attention over a T x H x W grid of video tokens
 * (plus optional trailing text tokens) in which every head only attends to a
 * per-head set of space-time tiles.  The kept set follows Sec. 4.1 of the paper:
 * frames are grouped by their distance from the query's frame, and inside each
 * group the spatial mask is the union of two query-centred windows (Eq. 1 is one
 * window, Eq. 2 the union of two, a window as large as the grid is the global
 * pattern of Sec. 3.2).  The mask is built once, offline (Sec. 3.3), and the
 * attention pass visits only kept tiles with an online softmax (Appendix D).
 *
 * Conventions common to every entry point
 *   - Plain C, no exceptions; every function that can fail returns a ca_status
 *     (0 = success, negative = failure) and records a message readable through
 *     compact_attn_last_error() on the calling thread.
 *   - "device pointer" = memory of the current HIP device, owned by the caller,
 *     16-byte aligned.  "host pointer" = ordinary process memory.
 *   - Tensors are contiguous [batch, num_heads, N, head_dim], element type
 *     ca_problem.dtype.  N = N_real (natural order) or N_pad (tile order), see below.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Compute
 *     calls enqueue work on it and return without synchronising, with one exception: the first
 *     compute call that uses a layout not yet passed to compact_attn_layout_upload allocates and
 *     copies that layout's device tables synchronously (and fails with CA_ERR_INVALID_ARG if
 *     `stream` is being captured at that moment).
 *   - A layout may be used by compute calls on several streams at once; launches of 4096 rows and
 *     more keep a ticket counter in the layout's device tables while they run, one of 64 taken
 *     round-robin at the call, so at most 64 such launches of one layout may be in flight on
 *     different streams at a time (launches on one stream run one after the other and never
 *     conflict).  A call captured into a HIP graph keeps the counter it was given: replays of that
 *     graph must not overlap in time with other launches of the same layout on other streams
 *     (build a second layout for those).
 *   - Failures detected on the host leave all outputs untouched.
 *
 * Tile arithmetic (Sec. 4.1, space-time tiles; Sec. 3.1 / Appendix D, tile-order flattening)
 *   tile = tt x th x tw tokens, B = tt*th*tw; tile grid nT = ceil(T/tt), nH = ceil(H/th),
 *   nW = ceil(W/tw); n_vid = nT*nH*nW video tiles followed by n_txt = n_text/B text tiles;
 *   n = n_vid + n_txt; N_real = T*H*W + n_text; N_pad = n*B.
 *   Natural order: token (t,y,x) at (t*H + y)*W + x, text tokens after the video tokens.
 *   Tile order: token (t,y,x) at tile*B + slot with tile = ((t/tt)*nH + y/th)*nW + x/tw and
 *   slot = ((t%tt)*th + y%th)*tw + x%tw; text token j at n_vid*B + j.  Slots of a tile that
 *   fall outside the grid are padding: zero on input, never attended, zero on output.
 */
#ifndef COMPACT_ATTN_H
#define COMPACT_ATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CA_OK = 0,
  CA_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, malformed head description, misalignment */
  CA_ERR_UNSUPPORTED = -2, /* valid request the device kernels do not cover (see compact_attn_forward)   */
  CA_ERR_ALLOC = -3,       /* host or device allocation failed                                          */
  CA_ERR_HIP = -4          /* a HIP runtime call or kernel launch failed; message carries the HIP text  */
} ca_status;

typedef enum { CA_F32 = 0, CA_BF16 = 1 } ca_dtype;

/* Pattern families a window search may use (the three columns of Table 3), each containing the one
 * before: a cubic window (one spatial window for every kept frame distance plus a temporal radius),
 * one window per frame group (Sec. 4.1, frame-group-wise patterns), two windows per frame group
 * (Sec. 4.1, dual attention windows). */
typedef enum { CA_PATTERN_CUBIC = 0, CA_PATTERN_FRAME_GROUPS = 1, CA_PATTERN_DUAL = 2 } ca_pattern;

/* One axis-aligned, query-centred window in tile units: key tile (kh,kw) is inside iff
 * |kh-qh| <= rh and |kw-qw| <= rw (Eq. 1).  A negative radius marks the window absent. */
typedef struct {
  int32_t rh, rw;
} ca_window;

/* One frame-distance group (Sec. 4.1, frame-group-wise patterns): applies to key tiles whose
 * tile-frame distance |kt-qt| is <= max_dt and larger than the previous group's max_dt.
 * Kept iff inside window a or window b (Sec. 4.1, dual attention windows; Eq. 2). */
typedef struct {
  int32_t max_dt;
  ca_window a, b;
} ca_group;

/* One head: up to CA_MAX_GROUPS groups, max_dt non-negative and strictly increasing.
 * Key tiles farther than the last group's max_dt are dropped.  num_groups = 0 keeps only text tiles.
 * clamp_centre = 0: windows are centred on the query tile and clipped by the grid (Eq. 1 as written).
 * clamp_centre = 1: a window keeps its full size at the border, the way sliding-tile windows do: on an
 * axis of L tiles a window of radius r with 2r+1 < L is centred at min(max(q, r), L-1-r) instead of q,
 * and a window with 2r+1 >= L covers the whole axis. */
#define CA_MAX_GROUPS 8
typedef struct {
  int32_t num_groups;
  int32_t clamp_centre;
  const ca_group* groups; /* host pointer, read during compact_attn_build_layout only */
} ca_head;

typedef struct {
  int32_t T, H, W;    /* video token grid                                      */
  int32_t tt, th, tw; /* tile shape                                            */
  int32_t n_text;     /* trailing text tokens, a multiple of B (0 = none)      */
  int32_t batch, num_heads, head_dim;
  int32_t dtype; /* ca_dtype                                                    */
  float scale;   /* softmax scale; <= 0 selects head_dim^-1/2                  */
} ca_problem;

typedef struct ca_layout ca_layout; /* opaque; immutable once built; may be shared by threads */

/* Build the sparse layout (Sec. 4.1; Sec. 3.3: masks are precomputed offline per head).
 *   problem  host pointer.  heads  host pointer to problem->num_heads descriptions.
 *   *out     receives a new layout owned by the caller (release with compact_attn_free_layout).
 * For every head and query tile the layout stores the ascending list of kept key-tile ids (CSR).
 * A text query tile keeps every tile; every query tile keeps all text tiles.  It also stores
 * the launch order of the (head, query tile) rows: descending kept count, ties by ascending
 * (head, tile).  Host-only work: no HIP call is made, so it also runs on a machine without a GPU.
 * Errors: CA_ERR_INVALID_ARG (null, non-positive dims, n_text not a multiple of B, bad groups),
 * CA_ERR_ALLOC. */
int compact_attn_build_layout(const ca_problem* problem, const ca_head* heads, ca_layout** out);

/* Import an arbitrary tile mask (Sec. 3.3: masks are precomputed offline; this is the door for masks
 * found by any search outside the library).
 *   row_ptr  host pointer to num_heads host pointers, each int64[n+1] (offsets into that head's col_idx).
 *   col_idx  host pointer to num_heads host pointers, each int32[row_ptr[h][n]]: kept key-tile ids of
 *            every query tile, strictly ascending inside a row, in [0, n).
 * The arrays are copied; nothing is added (no implicit text tiles): the mask is taken as given.
 * Errors: CA_ERR_INVALID_ARG (null, malformed problem, malformed CSR), CA_ERR_ALLOC. */
int compact_attn_layout_from_csr(const ca_problem* problem, const int64_t* const* row_ptr,
                                 const int32_t* const* col_idx, ca_layout** out);

/* Merge two layouts of the same problem by union, row by row (Sec. 4.2: configurations found for
 * different prompts are merged by union so that every region one of them needs is retained).
 * *out receives a new layout owned by the caller.  Errors: CA_ERR_INVALID_ARG (null, different
 * problems), CA_ERR_ALLOC. */
int compact_attn_layout_union(const ca_layout* a, const ca_layout* b, ca_layout** out);

/* Similarity of two binary tile masks (Eq. 3): |A and B| / |A or B| over the n x n tile pairs of head
 * head_a of a and head head_b of b; 1 when both are empty.  The layouts must have the same number of
 * tiles.  Errors: CA_ERR_INVALID_ARG. */
int compact_attn_layout_similarity(const ca_layout* a, int32_t head_a, const ca_layout* b, int32_t head_b,
                                   double* sim);

/* Sizes of a layout; any output pointer may be NULL. */
int compact_attn_layout_info(const ca_layout* layout, int64_t* n_tiles, int64_t* tokens_per_tile,
                             int64_t* n_tokens_real, int64_t* n_tokens_padded, int64_t* nnz_total);

/* Host views of one head's CSR, owned by the layout and valid until it is freed:
 *   *row_ptr -> int64[n+1] offsets into *col_idx, relative to this head;
 *   *col_idx -> int32[(*row_ptr)[n]] kept key-tile ids, ascending inside each row. */
int compact_attn_layout_csr(const ca_layout* layout, int32_t head, const int64_t** row_ptr,
                            const int32_t** col_idx);

/* Host view of the work ordering of all rows: int32[num_heads*n] of row ids head*n + query_tile by
 * descending number of kept key tiles, ties by ascending row id.  It is the launch order of the
 * kernels that give every row a workgroup of its own; where two query tiles share a workgroup see
 * compact_attn_layout_pairs and compact_attn_layout_packing. */
int compact_attn_layout_order(const ca_layout* layout, const int32_t** order);

/* Host view of the workgroups that serve two query tiles (work ordering of Appendix D's block loop
 * when a workgroup walks the union of two kept lists; bf16, head_dim 128):
 *   *pairs -> int32[2 * *num_pairs]; entries 2i and 2i+1 are row ids head*n + query_tile of the two
 *   tiles of workgroup i (same head), the second -1 when there is only one.
 *   64-token tiles: every row of the layout is in exactly one pair: neighbours along one grid axis
 *   chosen per head so that the unions are smallest; text tiles pair in id order.
 *   128-token tiles: only query tiles on a padded face of the grid, whose tokens fill fewer than four
 *   32-query waves, are here: their waves are packed along w, four to a workgroup, so a tile may
 *   appear in two consecutive workgroups with different waves (compact_attn_layout_packing), and only
 *   in heads where packing is cheaper than a workgroup per tile.
 *   Workgroups are in launch order: descending union size, ties in the order (head, first tile id).
 *   *walk_ptr -> int64[*num_pairs + 1] offsets into *walk;  *walk -> int32 words, for workgroup i the
 *   union of its two rows in ascending key-tile order, each word = tile id (bits 0-23)
 *   | 1 << 30 if the first tile's row keeps it | 1 << 31 if the second tile's row keeps it.
 * walk_ptr and walk may be NULL.  *num_pairs is 0 for layouts without such workgroups.
 * Owned by the layout, valid until it is freed. */
int compact_attn_layout_pairs(const ca_layout* layout, const int32_t** pairs, int64_t* num_pairs,
                              const int64_t** walk_ptr, const int32_t** walk);

/* Host view of how the launch is divided between the kernels:
 *   *desc -> int32[num_pairs] (num_pairs of compact_attn_layout_pairs), one word per workgroup of two
 *   query tiles: bit w (w = 0..3): wave w works for the second tile (else the first); bit 4 + w: wave
 *   w has queries at all; bits 8 + 4w .. 11 + 4w: the first of the wave's 32 query slots, divided by
 *   32, in the order that lists a tile's token-holding slots first.
 *   *launch_rows -> int32[*num_launch_rows]: the launch order of the kernel that gives a row a
 *   workgroup of its own, longest list first: an entry >= 0 is a row id head*n + query_tile (these
 *   are compact_attn_layout_order without the rows of packed tiles, in the same order), an entry
 *   e < 0 stands for workgroup ~e of compact_attn_layout_pairs, which the same launch runs (128-token
 *   tiles).  *num_launch_rows is 0 (and *launch_rows NULL) when every row is in a pair (64-token tiles).
 * Every query slot that holds a token belongs to exactly one wave of one workgroup.  Owned by the
 * layout, valid until it is freed. */
int compact_attn_layout_packing(const ca_layout* layout, const int32_t** desc, const int32_t** launch_rows,
                                int64_t* num_launch_rows);

/* Copy the layout's device-side tables (CSR, order, padding masks) to the current HIP device.
 * Synchronous; idempotent.  The compute calls below do it on first use if it was not called
 * (not possible while their stream is being captured).
 * Errors: CA_ERR_ALLOC, CA_ERR_HIP. */
int compact_attn_layout_upload(ca_layout* layout);

/* Release a layout and its device tables (NULL is ignored).  The caller must make sure no
 * enqueued work still reads it. */
void compact_attn_free_layout(ca_layout* layout);

/* Tile-order flattening (Sec. 3.1, Appendix D) and its inverse; device pointers.
 *   inverse = 0: src [batch, heads, N_real, D] natural order -> dst [batch, heads, N_pad, D]
 *                tile order; padding slots of dst are written as zero.
 *   inverse = 1: src [.., N_pad, D] tile order -> dst [.., N_real, D] natural order.
 * src and dst must not overlap.  Bit-exact copy of the elements. */
int compact_attn_permute(const void* src, void* dst, ca_layout* layout, int32_t inverse, void* stream);

/* Sparse attention forward (Appendix D: block-wise pass with online softmax over kept tiles).
 *   q, k, v, out: device pointers, [batch, heads, N_pad, D] in tile order; padding slots of
 *   k and v are ignored, padding rows of out are written as zero.  out must not overlap q/k/v
 *   (byte ranges of the whole tensors are compared).
 * For each query tile i of each head:  out_i = softmax(scale * Q_i K_J^T) V_J, J = real tokens of
 * the kept key tiles.  A row whose kept set holds no real key yields zeros.
 * bf16 problems run on the MFMA kernel: bf16 operands, fp32 accumulation and softmax state,
 * probabilities rounded to bf16 before the PV product; supported (B, D): (64,64), (64,128),
 * (128,128) and (128,64).  f32 problems run on a plain fp32 kernel for B <= 128, D in {32,64,128}.
 * Anything else: CA_ERR_UNSUPPORTED. */
int compact_attn_forward(const void* q, const void* k, const void* v, ca_layout* layout, void* out,
                         void* stream);

/* compact_attn_forward for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result, bit for bit, but the layout's tables (row offsets, packed tile words, launch order, padding
 * masks, pair walks) are read from a fixed 8 MiB device array inside the library instead of from
 * memory allocated at compact_attn_layout_upload; the call makes no hipMalloc / hipFree and needs no
 * prior upload.  Every GPU the library runs on holds one such array until the process ends.
 *   - A layout whose tables exceed the array (about 1.9 million kept tile pairs) is rejected with
 *     CA_ERR_UNSUPPORTED and a message that states both sizes; nothing is enqueued.
 *   - The array keeps the tables of the layout the previous call on this GPU used.  A call with the
 *     same layout enqueues the kernel only; a call with another layout first enqueues one
 *     host-to-device copy of that layout's tables on `stream` (the layout must stay alive until that
 *     copy has run).  Such a copy cannot be recorded into a capturing stream: make one call with
 *     the layout before the capture, otherwise CA_ERR_INVALID_ARG.
 *   - All calls on one GPU share the array: calls that may overlap in time on different streams
 *     race and must be ordered by the caller. */
int compact_attn_forward_static(const void* q, const void* k, const void* v, ca_layout* layout, void* out,
                                void* stream);

/* The same forward on tensors in NATURAL token order (Sec. 3.1's tile-wise flattening and its inverse
 * folded into the attention pass: the kernel gathers the K/V tiles and the Q rows from natural
 * order and scatters the output rows back, so no compact_attn_permute pass is needed).
 *   q, k, v, out: device pointers, [batch, heads, N_real, D] in natural order; out must not alias
 *   q/k/v.  Every row of out is written (zeros for a query whose kept set holds no real key).
 * Same arithmetic per query as compact_attn_forward, bit for bit, provided k and v hold finite
 * values: the padding slots of edge tiles, which the tile-order tensors hold as zeros, alias other
 * rows of the tensor here and enter the products with weight zero.  Supported: bf16 with (B, D) as for
 * compact_attn_forward and a tile width tw that is a multiple of 1024 / (2*D) tokens (4 for D = 128,
 * 8 for D = 64); otherwise CA_ERR_UNSUPPORTED. */
int compact_attn_forward_natural(const void* q, const void* k, const void* v, ca_layout* layout, void* out,
                                 void* stream);

/* Same kernel with every query tile keeping all n tiles (the full-attention starting point of
 * Sec. 4.2 and the baseline of Sec. 5.1); the per-head windows of the layout are ignored. */
int compact_attn_dense(const void* q, const void* k, const void* v, ca_layout* layout, void* out,
                       void* stream);

/* Attention mass per tile pair (Sec. 4.2: masks are searched by the recall they keep, the share of
 * the full attention's probability mass that falls on kept tile pairs).
 *   q, k   device pointers, [batch, heads, N_pad, D] in tile order (as for compact_attn_forward).
 *   mass   device pointer, float32 [batch, heads, n, n], written in full:
 *          mass[b, h, a, c] = sum over real query tokens i of tile a and real key tokens j of tile c of
 *          softmax_j(scale * q_i . k_j), the softmax taken over ALL real keys (full attention; the
 *          windows of the layout are ignored, only its geometry and scale are used).
 * Row a of mass sums to the number of real tokens of tile a.  One Q K^T product per tile pair: half
 * the FLOPs of one dense pass.
 *   Workspace: the kernel keeps two floats per (query token, key tile) of the rows in flight.  The
 *   first call for a layout allocates min(batch * heads * n, W) * N_pad * 8 bytes of device memory,
 *   W = the workgroups the device holds at a time (two per compute unit for 128-token tiles, four
 *   for 64-token tiles: 0.54 GB for 130K tokens on 256 compute units), (synchronously; refused with CA_ERR_INVALID_ARG on a stream under capture: call once
 *   before capturing), which the layout owns until compact_attn_free_layout.  Calls on the same
 *   layout that overlap in time (different streams) would share that workspace and race: give
 *   concurrent calls a layout each.  CA_ERR_ALLOC if the allocation fails.
 * Supported: bf16 with (B, D) in {64,128} x {64,128}; otherwise CA_ERR_UNSUPPORTED. */
int compact_attn_tile_mass(const void* q, const void* k, ca_layout* layout, float* mass, void* stream);

/* Window search of one head by boundary contraction (Sec. 4.2), host only.
 *   layout         any layout of the problem (only its geometry is used).
 *   mass           host pointer, float32 [n*n]: one head's attention mass per tile pair, row-major
 *                  (query tile, key tile), e.g. one [n, n] slice of compact_attn_tile_mass copied back.
 *   group_max_dt   host pointer, num_groups frame-distance boundaries (non-negative, strictly increasing;
 *                  tile-frame distances beyond the last are dropped, as in ca_head).
 *   tau, lambda    recall must stay >= tau; a contraction step whose (delta recall / delta cost) exceeds
 *                  lambda is not taken.  Recall and cost are fractions of the head's video-to-video mass
 *                  and tile pairs (text tiles are always kept and take no part).
 *   pattern        ca_pattern: CA_PATTERN_DUAL searches two windows per group as described below;
 *                  CA_PATTERN_FRAME_GROUPS one window per group (no notch steps: window b is always
 *                  absent); CA_PATTERN_CUBIC one window shared by the groups 0..k-1 and the groups from
 *                  k on dropped (steps: lower or narrow the shared window, drop the outermost kept
 *                  group; with boundaries 0, 1, 2, ... this is a sliding cube of tiles).
 *   groups         host pointer, receives num_groups groups (max_dt as given, windows found; both windows
 *                  absent = the group is dropped), ready to be put in a ca_head.
 *   recall, kept_fraction   optional outputs: recall and share of video-to-video tile pairs kept.
 * Starting from full coverage, each group's kept region on folded offsets (|dh|, |dw|) is a box with a
 * notch at its far corner, i.e. the union of a wide and a tall window (Eq. 2); the cheapest admissible
 * step over all groups (lower / narrow the box, open / deepen / widen the notch, drop the group) is
 * applied until none is left.  The groups shrink independently, each on its own masses, but share the
 * one recall budget tau of the head.  A mass whose video-to-video part sums to zero returns full
 * coverage (recall 1): there is nothing to rank steps by.  Errors: CA_ERR_INVALID_ARG (null, bad
 * groups or thresholds, a negative or non-finite mass entry), CA_ERR_ALLOC. */
int compact_attn_search_head(const ca_layout* layout, const float* mass, const int32_t* group_max_dt,
                             int32_t num_groups, double tau, double lambda, int32_t pattern, ca_group* groups,
                             double* recall, double* kept_fraction);

/* Message of the last failure on the calling thread ("" if none); valid until the next call. */
const char* compact_attn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* COMPACT_ATTN_H */
