/*
 * clear_attn.h -- C ABI of the MI355X (gfx950) CLEAR local attention: forward pass, backward pass, row bands.
 *
 * The operation (arXiv 2412.16112): softmax attention of Eq. 1 (Sec. 2),
 *     O = softmax(Q K^T / sqrt(head_dim)) V,
 * restricted to the pairs allowed by the mask of Eq. 3 (Sec. 3.2): a text query attends to every
 * key; an image query attends to every text key and to the image keys whose squared Euclidean
 * distance on the gridH x gridW token raster is strictly below r^2.  The window is cut off at the
 * image border (no wrap-around, no shifting) -- the reading that reproduces the FLOP counts of
 * Tables 2, 3 and 7.
 *
 * Tensor layout (all entry points): Q, K, V, O are DEVICE pointers to contiguous
 * [B, H, N, head_dim] arrays, N = n_text + gridH*gridW.  Rows 0 .. n_text-1 of the N axis are the
 * text tokens; row n_text + y*gridW + x is image token (y, x), raster order.  Base pointers must be
 * 16-byte aligned; O must not overlap Q, K or V.  Inputs are taken as given (post-RoPE); the only
 * scaling applied is 1/sqrt(head_dim).  Values must be finite.
 *
 * Supported: dtype CLEAR_BF16 with head_dim 128 or 64 (MFMA path; fp32 accumulation, one round-to-nearest
 * -even to bf16 on output) and dtype CLEAR_F32 with head_dim 64 (plain fp32 accuracy path).
 * n_text >= 0, gridH, gridW >= 1 (at most 32767 each), r >= 1.  bf16 contexts need N < 2^24 (the kernels address
 * one head with 32-bit byte offsets) and clear_attn_create refuses more with CLEAR_ERR_UNSUPPORTED, as it refuses
 * a tile schedule of more than 2^31 - 1 (query tile, key tile) pairs (r close to the grid size on a large grid);
 * fp32 contexts need N < 2^31.  Offsets across heads and batch items are 64-bit.
 *
 * Errors: every function returns a clear_status; nothing throws or aborts; invalid arguments are
 * rejected before any device work.  clear_attn_last_error gives a human-readable reason.
 * Thread safety: a context may be used by one thread at a time; distinct contexts are independent.  Calls on one
 * context share its workspaces, so they must be ordered among themselves: enqueue them on one stream, or make the
 * later call's stream wait for the earlier call; use one context per stream for concurrent calls.
 * All functions run on the current HIP device; a context belongs to the device current at create.
 * Streams: every call enqueues all of its work on the stream passed in, and on no other; the work is complete when
 * that stream has reached the end of it.
 */
#ifndef CLEAR_ATTN_H
#define CLEAR_ATTN_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct clear_attn_ctx clear_attn_ctx; /* opaque, owned by the library */

typedef enum {
    CLEAR_OK = 0,
    CLEAR_ERR_INVALID_ARG = 1, /* NULL pointer, non-positive size, r < 1, misaligned pointer */
    CLEAR_ERR_UNSUPPORTED = 2, /* (dtype, head_dim) pair without a kernel */
    CLEAR_ERR_ALLOC = 3,       /* host or device allocation failed */
    CLEAR_ERR_HIP = 4,         /* a HIP runtime call failed; see clear_attn_last_error */
    CLEAR_ERR_MISMATCH = 5     /* forward() shape arguments differ from those given to create() */
} clear_status;

typedef enum { CLEAR_BF16 = 0, CLEAR_F32 = 1 } clear_dtype;

#define CLEAR_TILE_PARTIAL 0 /* some slot pair of the two tiles is masked or outside the grid */
#define CLEAR_TILE_FULL 1    /* every slot pair is inside the grid and unmasked */

/*
 * Builds the tile schedule for (gridH, gridW, r) with the tile shapes of the kernel chosen for
 * (dtype, head_dim), and uploads it.  Allocates device memory and synchronises the device.
 * *out is written only on CLEAR_OK.  (Schedule: Sec. 3.2 fixes which pairs exist; the tiling is
 * this library's.)
 */
int clear_attn_create(clear_attn_ctx** out, int n_text, int gridH, int gridW, int head_dim, int r,
                      int dtype);

/*
 * Pre-sizes the workspace that the text-query rows need (partial results of the key-split dense
 * pass; text-query rows are dense over all tokens, Sec. 3.2, Eq. 3) for batch*heads = BH.
 * forward() calls this itself when it meets a larger B*H than any before, which allocates and
 * synchronises; call reserve first if forward must not allocate.  A forward call (any variant, backward
 * included) that would have to grow a workspace while `stream` is being captured into a HIP graph returns
 * CLEAR_ERR_INVALID_ARG instead and launches nothing: reserve beforehand, or make one eager call first.  Every
 * call launches on `stream` alone.
 * Returns CLEAR_ERR_ALLOC on failure.
 */
int clear_attn_reserve(clear_attn_ctx* ctx, int BH);

/*
 * Enqueues one forward pass (Eq. 1 under the mask of Eq. 3) on `stream` (a hipStream_t; NULL is
 * the default stream) and returns without synchronising.  n_text, gridH, gridW, head_dim, r must
 * equal the values given to create (CLEAR_ERR_MISMATCH otherwise, nothing launched).  B, H >= 1.
 * The caller owns Q, K, V, O and the stream, and must keep them alive until the stream has
 * finished the work.  Two forwards of one context may not overlap in time (shared workspace).
 */
int clear_attn_forward(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O,
                       int B, int H, int n_text, int gridH, int gridW, int head_dim, int r,
                       void* stream);

/*
 * clear_attn_forward for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, checks and results as clear_attn_forward, but
 * it calls no hipMalloc / hipFree and no allocating library routine: the key-split partial results of the
 * text-query rows go to a static device array of the library (112 MiB per GPU, held until the process ends)
 * instead of the context's workspace.
 * A call whose partial results (B*H * key splits * n_text * (head_dim + 2) floats) do not fit the array returns
 * CLEAR_ERR_UNSUPPORTED with the sizes in clear_attn_last_error, and launches nothing; the FLUX-8K shape (B*H = 24,
 * 16 splits, 512 text tokens, head_dim 128: 102 MB) fits.  The context's device must be the current one.
 * Every call on a GPU, from any context, shares that GPU's array: calls that overlap in time on one GPU race;
 * order them on one stream or with events.  Nothing in the array has to be cleared between calls.
 */
int clear_attn_forward_noalloc(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O,
                               int B, int H, int n_text, int gridH, int gridW, int head_dim, int r,
                               void* stream);

/*
 * Timing aid for benchmarks: same arguments and checks as clear_attn_forward, but runs `reps`
 * (1..256) forward passes back to back on `stream` with a HIP event between the kernels, and
 * SYNCHRONISES.  phase_ms[0..2] receive the average milliseconds per launch, inside that sequence,
 * of (0) the image-query kernel (Eq. 3's windowed rows), (1) the text-query kernel (dense rows,
 * split along the keys) and (2) the merge of those splits.  O holds a valid result afterwards.  The three
 * kernels are launched one by one here also for the problem sizes at which clear_attn_forward sends the first two
 * out as one launch (same code, same key splits, same bits).
 */
int clear_attn_forward_profile(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V,
                               void* O, int B, int H, int n_text, int gridH, int gridW,
                               int head_dim, int r, void* stream, int reps, float* phase_ms);

/* Frees the context and its device memory.  NULL is a no-op.  The caller must have synchronised
 * any stream still running a forward of this context. */
void clear_attn_destroy(clear_attn_ctx* ctx);

/* ---- introspection (host only, no device work) -------------------------------------------- */

/* sum(M) of Eq. 3 per (batch, head) from a lattice-point count; the FLOP estimate of the paper
 * (Fig. 2 caption) is 4 * sumM * channels. */
int clear_attn_mask_count(int n_text, int gridH, int gridW, int r, unsigned long long* sumM);

/* Tile shapes used for (dtype, head_dim): query tiles q_tile_h x q_tile_w and key tiles
 * k_tile_h x k_tile_w, both aligned to the grid origin and numbered row-major. */
int clear_attn_tile_shape(int head_dim, int dtype, int* q_tile_h, int* q_tile_w, int* k_tile_h,
                          int* k_tile_w);

/*
 * Host-only schedule builder.  For each query tile (row-major) the ascending list of key tiles
 * holding at least one in-grid, unmasked (query, key) image pair, with CLEAR_TILE_FULL /
 * CLEAR_TILE_PARTIAL flags.  Text keys are attended by every query and are not listed.
 * Call once with row_ptr = col_idx = flags = NULL to get *n_q_tiles and *n_pairs, then with
 * caller-owned arrays row_ptr[*n_q_tiles + 1], col_idx[*n_pairs], flags[*n_pairs].
 */
int clear_attn_schedule_host(int gridH, int gridW, int r, int q_tile_h, int q_tile_w, int k_tile_h,
                             int k_tile_w, int* n_q_tiles, long long* n_pairs, int* row_ptr,
                             int* col_idx, unsigned char* flags);

/* The schedule a context holds (same content as clear_attn_schedule_host for its tile shapes). */
int clear_attn_schedule_size(const clear_attn_ctx* ctx, int* q_tile_h, int* q_tile_w, int* k_tile_h,
                             int* k_tile_w, int* n_q_tiles, long long* n_pairs);
int clear_attn_schedule_copy(const clear_attn_ctx* ctx, int* row_ptr, int* col_idx,
                             unsigned char* flags);

/* Number of (query slot, key slot) pairs per (batch, head) that the kernels actually push through
 * the matrix pipeline, masked and padding slots included ("executed" work; useful work is sumM). */
int clear_attn_executed_pairs(const clear_attn_ctx* ctx, unsigned long long* pairs_per_head);

/* ---- Other local masks through the same scheduler (the sparse-attention variants the paper compares CLEAR
 * with; the text rule of Eq. 3 - text rows and columns all ones - is kept for every kind):
 *   CLEAR_MASK_DISC    dx^2 + dy^2 < r^2 (Eq. 3; what clear_attn_create builds)
 *   CLEAR_MASK_SQUARE  |dx| < r and |dy| < r: a (2r-1) x (2r-1) window centred on the query, cut off at the border
 *   CLEAR_MASK_SWIN    both tokens in the same r x r window of the partition whose origin is moved up and left
 *                      by `shift` (0 <= shift < r; the windows cut by the border are smaller); shift 0 and r/2
 *                      on alternate layers give the shifted-window scheme
 *   CLEAR_MASK_STRIDED the key's offset from the query (key minus query), modulo r on each axis with a non-negative
 *                      remainder, equals (l % r, (l / r) % r); the layer index l >= 0 is passed as `shift`.  Each
 *                      query sees one key per r x r cell.  bf16 only, gridH >= r and gridW >= r; forward (with or
 *                      without prologue, with or without lse) and backward, no row bands.  It runs as r*r dense problems, one per residue class (y % r, x % r) of the
 *                      queries, with strided token addresses; the context's tile schedule (clear_attn_schedule_size /
 *                      _copy) is that of one class, a ceil(gridH / r) x ceil(gridW / r) grid; clear_attn_schedule_
 *                      host_masked returns CLEAR_ERR_UNSUPPORTED for it.
 * Every other entry point takes a square or Swin context unchanged (forward, forward_band, backward, ...); the
 * executed work differs: the square window has precomputed lane masks like the disc; Swin windows run whole or
 * skipped blocks when r and shift are multiples of 8 and the arithmetic element mask otherwise. */
typedef enum { CLEAR_MASK_DISC = 0, CLEAR_MASK_SQUARE = 1, CLEAR_MASK_SWIN = 2, CLEAR_MASK_STRIDED = 3 } clear_mask_kind;
int clear_attn_create_masked(clear_attn_ctx** out, int n_text, int gridH, int gridW, int head_dim, int r,
                             int dtype, int mask_kind, int shift);
/* clear_attn_schedule_host for a mask kind. */
int clear_attn_schedule_host_masked(int gridH, int gridW, int r, int mask_kind, int shift, int q_tile_h, int q_tile_w,
                                    int k_tile_h, int k_tile_w, int* n_q_tiles, long long* n_pairs, int* row_ptr,
                                    int* col_idx, unsigned char* flags);
/* sumM for a mask kind (clear_attn_mask_count is the disc). */
int clear_attn_mask_count_masked(int n_text, int gridH, int gridW, int r, int mask_kind, int shift,
                                 unsigned long long* sumM);

/* ---- The block's query/key prologue fused into the forward pass (Sec. 3.1: the backbone perceives the two
 * image axes through a rotary position embedding; Sec. 4.3: its frequencies and a scale on the attention
 * logits are changed for resolution extrapolation).  bf16 only.
 *
 * Q and K are the raw projections; each token row x of a head goes through
 *   1. RMS normalisation, if its gain is non-NULL:  x_c * gain_c / sqrt(mean_c x_c^2 + norm_eps);
 *   2. rotary embedding, if rope_y and rope_x are non-NULL (both or neither): channels (2i, 2i+1) of the image
 *      token at (y, x) are turned by the sum of two angles given as (cos, sin) pairs, rope_y[y][i] and
 *      rope_x[x][i] (fp32, [gridH or gridW][head_dim/2][2]; a pair that an axis does not act on holds (1, 0)):
 *      (e, o) -> (cos e - sin o, sin e + cos o); text tokens are not turned;
 *   3. rounding to bf16,
 * and the softmax runs on logit_scale * q.k / sqrt(head_dim) (logit_scale > 0).  Gains are fp32 [head_dim];
 * all four tables are device pointers, 16-byte aligned, read-only, caller-owned.
 *
 * The query rows are transformed in registers as each workgroup loads them (no extra pass over Q); the key
 * rows, which many workgroups stage, are transformed once into a buffer the context owns (B*H*N*head_dim
 * bf16, allocated on first use or by clear_attn_reserve_prologue; K itself is not modified).  Errors as for
 * clear_attn_forward, plus CLEAR_ERR_UNSUPPORTED for an fp32 context. */
int clear_attn_forward_prologue(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, int B,
                                int H, int n_text, int gridH, int gridW, int head_dim, int r, const float* q_gain,
                                const float* k_gain, float norm_eps, const float* rope_y, const float* rope_x,
                                float logit_scale, void* stream);
int clear_attn_reserve_prologue(clear_attn_ctx* ctx, int BH);
/* Steps 1-3 on a whole tensor as a pass of its own: X, Y device bf16 [B, H, N, head_dim] (head_dim 64 or 128),
 * Y == X allowed, otherwise they must not overlap.  No context: errors are reported through the status and
 * clear_attn_last_error(NULL). */
int clear_attn_qk_prologue(const void* X, void* Y, int B, int H, int n_text, int gridH, int gridW, int head_dim,
                           const float* gain, float norm_eps, const float* rope_y, const float* rope_x,
                           void* stream);

/* ---- Tensors in another layout (the same operator as clear_attn_forward: Eq. 1 under the mask of Eq. 3).  Callers that cannot spare a transposing copy - Q, K, V straight out of a
 * projection as [B, N, H, head_dim], or slices of one packed [B, N, 3, H, head_dim] tensor, and O wanted the same
 * way - pass strides: `strides` points at 12 values, (batch, head, token) strides in elements for Q, K, V, O in this
 * order; element (b, h, n, c) of a tensor is at base + b*sb + h*sh + n*sn + c (channels contiguous).  bf16 contexts
 * only.  Every stride must be a multiple of 8 elements (base pointers 16-byte aligned as before), the token stride
 * >= head_dim, the others >= 0 (an input may repeat over heads or batch; O's must be > 0); K and V are addressed
 * with 32-bit byte offsets inside a head, so N * token stride * 2 must stay below 2^32; O's address range must not
 * overlap an input's.  Same results, bit for bit, as the plain layout.  lse of clear_attn_forward_strided: NULL, or
 * where to write the log-sum-exp of clear_attn_forward_lse (always the plain [B, H, N] fp32 layout).  The row-band
 * entry points take the plain layout only.
 * clear_attn_backward_strided: clear_attn_backward with 24 stride values, for Q, K, V, O, dO, dQ, dK, dV in this order;
 * the same rules, with Q, K, V, dO under the 32-bit limit and dQ, dK, dV in the place of O. */
int clear_attn_forward_strided(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, float* lse,
                               const long long* strides, int B, int H, int n_text, int gridH, int gridW, int head_dim,
                               int r, void* stream);
int clear_attn_backward_strided(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, const void* O,
                                const void* dO, const float* lse, void* dQ, void* dK, void* dV, const long long* strides,
                                int B, int H, int n_text, int gridH, int gridW, int head_dim, int r, void* stream);
int clear_attn_forward_prologue_strided(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O,
                                        const long long* strides, int B, int H, int n_text, int gridH, int gridW,
                                        int head_dim, int r, const float* q_gain, const float* k_gain, float norm_eps,
                                        const float* rope_y, const float* rope_x, float logit_scale, void* stream);

/* ---- Training: forward with the softmax statistics, and the backward pass (the attention layers are the
 * trained parameters of the distillation of Sec. 3.3; the gradients follow from differentiating Eq. 1
 * under the mask of Eq. 3).  bf16 only (head_dim 128 or 64).
 *
 * clear_attn_forward_lse: clear_attn_forward that also writes, for every row, the natural logarithm of its
 * softmax denominator sum_j exp(q_i.k_j / sqrt(head_dim)) over the attended keys to lse (device, fp32,
 * [B, H, N], caller-owned). */
int clear_attn_forward_lse(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, float* lse,
                           int B, int H, int n_text, int gridH, int gridW, int head_dim, int r, void* stream);

/* Backward pass.  Q, K, V as given to the forward pass, O and lse as it returned them, dO the gradient with
 * respect to O; writes dQ, dK, dV (device, [B, H, N, head_dim], the tensors' dtype; fp32 accumulation, one
 * rounding on output).  All tensors 16-byte aligned; dQ, dK, dV must not overlap each other or an input.
 * Enqueues on stream, never synchronises; allocates only if the context's backward workspace ([B*H][N] floats
 * plus the split sums of the text rows) has to grow: call clear_attn_reserve_backward beforehand to avoid
 * that.  Shape arguments as for clear_attn_forward (CLEAR_ERR_MISMATCH otherwise, nothing launched). */
int clear_attn_backward(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, const void* O,
                        const void* dO, const float* lse, void* dQ, void* dK, void* dV, int B, int H, int n_text,
                        int gridH, int gridW, int head_dim, int r, void* stream);
int clear_attn_reserve_backward(clear_attn_ctx* ctx, int BH);

/* ---- Row bands: patch-parallel inference, one band of image rows per GPU (multi-GPU section, Eq. 7) ----
 *
 * The gridH_total x gridW feature map is cut into n_bands bands of whole rows.  A band is processed
 * with a context created for its LOCAL grid: halo_top + (y1 - y0) + halo_bottom rows by gridW columns,
 * where the halo rows are copies of the r - 1 rows of K and V that the neighbouring bands hold next to the
 * cut (the only exchange the image tokens need).  The local tensors are laid out like any other:
 * [B, H, n_text + local_rows * gridW, head_dim], text tokens first.
 *
 * clear_attn_band_layout: rows [*y0, *y1) of band `band` of n_bands (as even as possible, larger bands
 * first) and the halo rows it needs on either side.  CLEAR_ERR_UNSUPPORTED when a band would be narrower
 * than its halo of r - 1 rows (the halo would have to come from beyond the adjacent band).  Host only. */
int clear_attn_band_layout(int gridH_total, int r, int n_bands, int band, int* y0, int* y1, int* halo_top,
                           int* halo_bottom);

/* Forward pass of one band.  ctx, Q, K, V, O, B .. r, stream: as for clear_attn_forward, for the local grid.
 * Image queries: only the rows [own_y0, own_y1) of the local grid are computed and written to O (exactly
 * their output in the undivided problem when the halo holds the r - 1 neighbouring rows, or more of them: rows
 * beyond r - 1 are out of every owned query's reach); halo rows of O are left untouched, and so are the text
 * rows.  The query tiles start at own_y0 itself, so no workgroup straddles the first owned row (bf16, disc mask,
 * own_y0 >= r - 1 as the halo of an inner band gives it; a band at the top of the image with fewer rows above
 * own_y0, the other masks and fp32 keep the tiles of the local grid, which start at row 0).  When own_y0 is not a
 * multiple of the query-tile height, the first call with that own_y0 (mod the tile height) builds tile lists of
 * its own: it allocates and waits for their upload, and is refused with CLEAR_ERR_INVALID_ARG while the stream is
 * being captured; later calls reuse them.
 * Text queries: attend to the owned image rows and, if text_keys != 0, to the text keys; the softmax output
 * over those keys goes to text_o (device, fp32, [B, H, n_text, head_dim]) and the natural logarithm of the
 * softmax denominator sum_j exp(q.k_j / sqrt(head_dim)) to text_lse (device, fp32, [B, H, n_text]); both
 * caller-owned, required when n_text > 0.  Combine the bands' results with clear_attn_merge_text.
 * Apart from that first call: never synchronises; allocates only if the text workspace has to grow (see
 * clear_attn_reserve). */
int clear_attn_forward_band(clear_attn_ctx* ctx, const void* Q, const void* K, const void* V, void* O, int B,
                            int H, int n_text, int gridH, int gridW, int head_dim, int r, int own_y0,
                            int own_y1, int text_keys, float* text_o, float* text_lse, void* stream);

typedef enum {
    CLEAR_MERGE_EXACT = 0,   /* weights exp(lse_p) / sum exp(lse_p): the softmax over the union of the bands' key
                                sets, exact when those sets are disjoint (text keys counted in one band only) */
    CLEAR_MERGE_AVERAGE = 1  /* Eq. 7: the plain mean of the per-band softmax outputs (each band: text keys and
                                its own image keys) */
} clear_merge_mode;

/* Combines n_parts (1..64) band results for the text rows and writes them, converted to dtype, into rows
 * 0 .. n_text-1 of every (batch, head) of O, a device [B, H, N, head_dim] tensor.  text_o, text_lse: HOST
 * arrays of n_parts DEVICE pointers as filled by clear_attn_forward_band (on several GPUs: after an
 * all-gather of these constant-size buffers).  Enqueues one kernel on stream; no allocation, no sync. */
int clear_attn_merge_text(int n_parts, const float* const* text_o, const float* const* text_lse, int B, int H,
                          int n_text, long long N, int head_dim, int mode, void* O, int dtype, void* stream);

/* Measurement aid (Sec. 1's FLOP accounting is quoted against the matrix peak): runs back-to-back
 * v_mfma_f32_32x32x16_bf16 on every SIMD of the current device for about `seconds` (0 < seconds <= 5)
 * and reports the sustained dense bf16 rate of the last launch in TFLOP/s and the shader clock it ran
 * at in MHz (host pointers, both required).  Synchronises the device; allocates and frees a few bytes. */
int clear_attn_measure_mfma_peak(double seconds, double* tflops, double* shader_mhz);

/* Reason of the last failure on this context (or of the last failed create when ctx is NULL).
 * The string is owned by the library and valid until the next call on the same context/thread. */
const char* clear_attn_last_error(const clear_attn_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* CLEAR_ATTN_H */
