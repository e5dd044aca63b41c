/*
 * toma.h -- C ABI of libtoma: one ToMA layer (Token Merge with Attention) on one AMD MI355X.
 *
 * The calls follow the paper's statement of the method (ToMA: Token Merge with Attention for
 * Diffusion Models): destinations are selected per local region by greedy facility location
 * (Sec. 4.1, Alg. 2), tokens are merged with an attention-like weight matrix (Sec. 4.2.1), a core
 * module runs on the merged tokens (here multi-head attention, Eq. 1), and the result is unmerged
 * by the transpose of the merge matrix (Sec. 4.2.2); Alg. 3 strings these together per region and
 * Sec. 4.3.2 reuses destinations and weights across steps.
 *
 * Conventions for every call
 *   - Data pointers are DEVICE pointers owned by the caller, 16-byte aligned, dense, row-major,
 *     last dimension contiguous.  Descriptors are host structs, read during the call only.
 *   - The library allocates nothing, frees nothing and never synchronises: all work is queued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and the call returns at
 *     once; outputs are valid after the caller synchronises the stream.
 *   - `ws` is caller-owned device scratch of at least toma_workspace_bytes() bytes, 256-byte
 *     aligned; its contents are undefined between calls.  Calls sharing one workspace must be
 *     ordered on one stream.
 *   - The return value is a toma_status.  Argument errors are found on the host before anything
 *     is launched; nothing is written in that case.  TOMA_ERR_LAUNCH reports a failed launch.
 *   - Tokens lie on a row-major H x W grid, token n = r*W + c.  Region p and local position l of a
 *     token: p = (r / tile_h) * (W / tile_w) + (c / tile_w), l = (r % tile_h) * tile_w + c % tile_w
 *     (tile-shaped regions, Sec. 4.3.1; tile_w == W gives stripe-shaped regions).
 *     P = regions per sample, N_loc = tile_h * tile_w, D = P * d_loc destinations per sample.
 *   - Values are expected to be finite.  The merge and unmerge products skip blocks of the stored
 *     weights that are entirely zero (with a small tau most of A is): a zero weight then contributes
 *     nothing even where 0 * inf or 0 * NaN would have contributed a NaN.  For finite inputs the
 *     results are those of the full products.
 *   - Limits: C % 32 == 0; N_loc % 16 == 0 and N_loc <= 2048 (regions of more than 256 tokens take a
 *     slower selection kernel that keeps the similarities in memory); 1 <= d_loc <= N_loc;
 *     merge_regions is 1 or P; head_dim is 32, 64 or 128.
 *     Anything else returns TOMA_ERR_UNSUPPORTED or TOMA_ERR_SHAPE.
 */
#ifndef TOMA_H
#define TOMA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TOMA_OK = 0,
  TOMA_ERR_NULL = 1,        /* a required pointer is NULL */
  TOMA_ERR_SHAPE = 2,       /* sizes are non-positive or do not divide as required */
  TOMA_ERR_ALIGN = 3,       /* a data pointer is not 16-byte aligned (workspace: 256) */
  TOMA_ERR_WORKSPACE = 4,   /* ws_bytes is smaller than toma_workspace_bytes() */
  TOMA_ERR_UNSUPPORTED = 5, /* a valid request outside the limits listed above */
  TOMA_ERR_LAUNCH = 6       /* the HIP runtime refused a launch */
} toma_status;

typedef enum { TOMA_F32 = 0, TOMA_BF16 = 1 } toma_dtype;

/* Shape of one layer call (inputs of Alg. 3: X in R^{B x N x d}, D, tau). */
typedef struct {
  int32_t B, H, W, C;    /* batch, grid height and width (N = H*W), channel width */
  int32_t tile_h, tile_w;/* region shape; must divide H and W */
  int32_t d_loc;         /* destinations kept per region */
  int32_t merge_regions; /* 1: merge weights over all tokens of a sample (the paper's "ToMA");
                            P: weights inside each region ("ToMA_tile", Alg. 3) */
  float tau;             /* merge temperature, > 0 */
  float logit_scale;     /* 0: use 1/tau (Sec. 4.2.1's display formula); else the multiplier */
  int32_t dtype;         /* toma_dtype of X, Xm, O, Y, the projection weights and A */
} toma_desc;

/* The core module: multi-head attention on [merged ; extra] tokens.  heads * head_dim == C.
 * t_extra tokens per sample (e.g. text tokens) join the attention unmerged. */
typedef struct {
  int32_t heads, head_dim, t_extra;
} toma_attn_desc;

/* Bytes of scratch any call with these descriptors needs (attn may be NULL for calls that take
 * no toma_attn_desc).  Returns 0 when the descriptors are invalid. */
size_t toma_workspace_bytes(const toma_desc *desc, const toma_attn_desc *attn);

/* Static string naming a status. */
const char *toma_status_string(int status);

/*
 * Destination selection (Sec. 4.1, Alg. 2; per region as in Alg. 3 step 1).
 * For every (sample, region): S_ij = cos(x_i, x_j) over the region's tokens; first pick = largest
 * row sum; every later pick maximises sum_j max(0, S_ij - m_j) over tokens not yet picked, with
 * m_j the largest similarity of token j to the picks so far.  Ties go to the lowest index.
 * Similarities are evaluated to double precision from the stored token values (bf16 tokens: exactly,
 * as integer sums on the int8 matrix cores; fp32 tokens: on the fp64 matrix cores) and rounded once
 * to the nearest multiple of 2^-30; the sums and comparisons over them are exact (64-bit integers),
 * so the picks do not depend on any summation order and mathematically tied candidates (frequent:
 * two tokens that only improve each other's coverage) are exact ties, decided by index alone.
 *   X        in   [B, N, C]         tokens (dtype)
 *   idx      out  [B, P, d_loc]     int32 grid index of each pick, in pick order
 *   gain_opt out  [B, P, d_loc]     float value of each winning candidate (the first: its row sum), or NULL
 *   gap_opt  out  [B, P, d_loc]     float lead of each winner over the best other candidate (0 = an
 *                                   exact tie, decided by index; +inf = no other candidate was left),
 *                                   or NULL.  gap / gain below 1e-6 marks a near tie.
 */
int toma_select(const toma_desc *desc, const void *X, int32_t *idx, float *gain_opt, float *gap_opt,
                void *ws, size_t ws_bytes, void *stream);

/*
 * toma_select for callers that cannot hand over or allocate a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid device allocation): the same selection, same
 * arguments and results, with its scratch (the regions' similarity matrices, B * P * N_loc^2 32-bit
 * words, and for bf16 tokens their fixed-point copy, 4 bytes per element) in a buffer of
 * TOMA_STATIC_SCRATCH_BYTES that is part of the library's device code and present once on every GPU.
 * No device memory is allocated or freed, at any call.
 *   - Shapes whose scratch exceeds the buffer return TOMA_ERR_WORKSPACE (the SDXL-sized layers fit:
 *     2 x 4096 tokens of width 640 need 8 + 20 MiB; the 128 x 128 grid does not).
 *   - The GPU the stream belongs to must be the current device of the calling thread.  The buffer's
 *     address on that GPU is looked up on the first call there (TOMA_ERR_LAUNCH if the runtime
 *     refuses).
 *   - All calls on one GPU share the one buffer: calls that may overlap in time on a GPU (different
 *     streams, different threads) race on it; order them.  Nothing in the buffer needs clearing
 *     between calls (every similarity that is read was written by the same call).
 */
#define TOMA_STATIC_SCRATCH_BYTES (32u << 20)
int toma_select_static(const toma_desc *desc, const void *X, int32_t *idx, float *gain_opt,
                       float *gap_opt, void *stream);

/*
 * Merge weights and merge (Sec. 4.2.1; Alg. 3 step 2).  Inside each merge region (all tokens
 * of the sample, or one region) with destinations j = rows idx of X and sources s:
 *   A_js = softmax over j of (logit_scale * <x_idx[j], x_s>)   per source s,
 *   Z_j  = sum_s A_js,   Xm_j = (1 / Z_j) * sum_s A_js x_s          (A~ = A / Z, Xm = A~ X)
 * Z_j is clamped below at 1e-20.  A is stored in dtype; Z sums the stored values of A.
 *   idx  in   [B, P, d_loc]             destinations (from toma_select or a cache)
 *   A    out  [B, R, D/R, N/R] dtype    R = merge_regions; sources in region order: source s of a
 *                                       merge region is token l = s % N_loc of its selection region
 *                                       s / N_loc (with R = P: of the region itself), so the tokens
 *                                       of one selection region are N_loc consecutive columns
 *   Z    out  [B, D] float
 *   amap out  toma_map_bytes(desc) bytes   block map of A (below); NULL iff toma_map_bytes(desc) == 0
 *   Xm   out  [B, D, C] dtype           merged tokens, rows in idx order
 * (A, Z, amap) is the cache that toma_merge_cached / toma_unmerge / toma_layer take: the three
 * belong together and are only valid with the descriptor they were written under; treat them as opaque.
 */
int toma_merge(const toma_desc *desc, const void *X, const int32_t *idx, void *A, float *Z, void *amap,
               void *Xm, void *ws, size_t ws_bytes, void *stream);

/*
 * The block map of a stored A (part of the pattern cache of Sec. 4.3.2).  With a small temperature
 * nearly every source token gives all of its weight to one or two destinations and the rest of its
 * column of A is stored as exact zeros; the map says, per block of 128 destinations x 32 sources of
 * every merge region, whether the block holds any nonzero value, and the merge and unmerge products
 * skip the blocks that do not.  Whoever writes A writes the map (toma_merge, toma_layer); it is
 * caller-owned device memory that lives as long as (A, Z) and must never outlive or be mixed with
 * another A: a map that marks an occupied block as empty silently drops that block's weights.
 *   toma_map_bytes   size of the map for this descriptor; 0 when the shape uses none (short
 *                    products), in which case every amap argument may be NULL
 *   toma_map_build   recomputes the map from an A that did not come out of this library's weight
 *                    kernels (restored from elsewhere, edited by the caller): one read of A
 */
size_t toma_map_bytes(const toma_desc *desc);
int toma_map_build(const toma_desc *desc, const void *A, void *amap, void *stream);

/* Merge with cached weights (Sec. 4.3.2): Xm = (A / Z) X for the CURRENT X and an (A, Z, amap)
 * computed earlier by toma_merge / toma_layer with the same descriptor. */
int toma_merge_cached(const toma_desc *desc, const void *X, const void *A, const float *Z,
                      const void *amap, void *Xm, void *ws, size_t ws_bytes, void *stream);

/*
 * Attention on the merged tokens (Eq. 1 with tau = 1; Alg. 3 "computational layer").
 * U = [Xm ; X_extra] (L = D + t_extra rows per sample); Q = U Wq, K = U Wk, V = U Wv; head h owns
 * channels [h*head_dim, (h+1)*head_dim); O_h = softmax(Q_h K_h^T / sqrt(head_dim)) V_h; heads are
 * concatenated; O = O Wo when Wo_opt is given.  Weights are [C, C] row-major, y = x W.
 *   Xm          in   [B, D, C]
 *   X_extra_opt in   [B, t_extra, C] (NULL iff t_extra == 0)
 *   O           out  [B, D + t_extra, C]
 */
int toma_attend(const toma_desc *desc, const toma_attn_desc *attn, const void *Xm,
                const void *X_extra_opt, const void *Wq, const void *Wk, const void *Wv,
                const void *Wo_opt, void *O, void *ws, size_t ws_bytes, void *stream);

/*
 * Cross-attention with the merged tokens as queries (Sec. 5.1: the ToMA_once variant merges once per
 * transformer block and runs every module of the block - self-attention, cross-attention, MLP - on
 * the merged tokens before one unmerge).  Eq. 1 with tau = 1 and separate token sets:
 * Q = U Wq; K = Ctx Wk, V = Ctx Wv; per head O_h = softmax(Q_h K_h^T / sqrt(head_dim)) V_h over the
 * context tokens; heads concatenated; O = O Wo when Wo_opt is given.
 *   U     in   [B, L, C]           L = D + attn->t_extra query tokens per sample (e.g. the output of
 *                                  toma_attend, or the merged tokens themselves)
 *   Ctx   in   [B, t_ctx, c_ctx]   context tokens (e.g. text embeddings); c_ctx % 32 == 0, t_ctx <= L
 *   Wq    in   [C, C];  Wk, Wv in [c_ctx, C];  Wo_opt in [C, C]   row-major, y = x W
 *   O     out  [B, L, C]           may not alias U
 */
int toma_cross_attend(const toma_desc *desc, const toma_attn_desc *attn, const void *U, const void *Ctx,
                      int32_t t_ctx, int32_t c_ctx, const void *Wq, const void *Wk, const void *Wv,
                      const void *Wo_opt, void *O, void *ws, size_t ws_bytes, void *stream);

/*
 * Transpose unmerge (Sec. 4.2.2; Alg. 3 step 3): Y[token(s)] = sum_j (A_js / Z_j) O_j for every
 * source s, written at the token's grid position (the region split is undone by addressing).
 *   O  in   [B, o_rows, C]   o_rows >= D; only rows [0, D) of each sample are read
 *   Y  out  [B, N, C]
 */
int toma_unmerge(const toma_desc *desc, const void *A, const float *Z, const void *amap, const void *O,
                 int32_t o_rows, void *Y, void *ws, size_t ws_bytes, void *stream);

/*
 * Merge and unmerge with the weights recomputed instead of stored (Sec. 4.2.1: the merge weights ARE
 * scaled dot-product attention, A = SDPA(X, D, I, tau), so A~ X and A~^T X' can be evaluated as
 * attention-shaped products without A ever existing in memory: useful where A is not reused across
 * steps, or is large - one merge region over a 128 x 128 grid stores half a gigabyte).
 *   toma_merge_recompute    Z_j = sum_s A_js and Xm_j = (1 / Z_j) sum_s A_js x_s with A_js evaluated on
 *                           the fly; also fills wcache
 *   toma_unmerge_recompute  Y[token(s)] = sum_j A_js O_j / Z_j for the SAME X and idx
 *   wcache  toma_recompute_cache_bytes(desc) bytes, 256-byte aligned, caller-owned, opaque: per source
 *           token the normaliser of its softmax over the destinations, and per (source, slice of
 *           destinations) the evidence by which tiles of weights that are entirely zero are skipped -
 *           O(N * D / 64) floats instead of A's N * D elements
 * Results agree with toma_merge / toma_unmerge to rounding (the weights enter the products rounded to
 * the element type here as there).  Limits: C <= 3072, at most 65536 tokens per merge region.
 */
size_t toma_recompute_cache_bytes(const toma_desc *desc);
int toma_merge_recompute(const toma_desc *desc, const void *X, const int32_t *idx, float *Z, void *wcache,
                         void *Xm, void *ws, size_t ws_bytes, void *stream);
int toma_unmerge_recompute(const toma_desc *desc, const void *X, const int32_t *idx, const float *Z,
                           const void *wcache, const void *O, int32_t o_rows, void *Y, void *ws,
                           size_t ws_bytes, void *stream);

/*
 * Moore-Penrose unmerge (Sec. 4.2.2, first display; the alternative the paper measures the transpose
 * against in App. E.4): Y[token(s)] = sum_j (A~^+)_sj O_j with A~ = A / Z the row-normalised merge
 * matrix of each merge region and A~^+ its pseudo-inverse, = A~^T (A~ A~^T)^-1 when the rows of A~ are
 * independent.  They often are not (a destination nobody chose is a zero row; near-duplicate
 * destinations give nearly dependent rows), so the pseudo-inverse is taken with a cut-off, as numerical
 * libraries do: singular values of A~ that are <= rcond * the largest count as zero.  The paper does not
 * name one; with tau = 0.1 the merge matrices of smooth inputs have a bulk of singular values in
 * [0.2, 1] and a few stragglers of 1e-4 and below, so 1e-2 separates them.
 * Computed in double precision from the stored A and Z (eigen-decomposition of A~ A~^T per region).
 *   rcond  in  0 <= rcond < 1
 *   O, Y   as for toma_unmerge
 * Limits: merge regions of at most 128 destinations (region-local merge at the usual sizes; one
 * merge region per sample only for small grids); otherwise TOMA_ERR_UNSUPPORTED.
 */
int toma_unmerge_pinv(const toma_desc *desc, const void *A, const float *Z, const void *O, int32_t o_rows,
                      float rcond, void *Y, void *ws, size_t ws_bytes, void *stream);

/*
 * One whole layer with pattern reuse (Alg. 3 + Sec. 4.3.2).  reuse_flags says what is taken from
 * the caller's cache instead of being recomputed from X:
 *   0                  select, weights, merge, attention, unmerge; idx, A, Z, amap are written
 *   TOMA_REUSE_IDX     idx is read; weights are recomputed; A, Z, amap are written
 *   TOMA_REUSE_A       idx is ignored, A, Z and amap are read (implies TOMA_REUSE_IDX)
 *   TOMA_RECOMPUTE_WEIGHTS   (alone or with TOMA_REUSE_IDX) no A is written or read: the merge and the
 *                      unmerge recompute the weights (toma_merge_recompute / toma_unmerge_recompute);
 *                      A and amap may be NULL; Z is written
 *   Y            out  [B, N, C]
 *   Y_extra_opt  out  [B, t_extra, C]  rows of O that belong to the extra tokens (NULL iff none)
 */
enum { TOMA_REUSE_IDX = 1, TOMA_REUSE_A = 2, TOMA_RECOMPUTE_WEIGHTS = 4 };
int toma_layer(const toma_desc *desc, const toma_attn_desc *attn, uint32_t reuse_flags,
               const void *X, const void *X_extra_opt, int32_t *idx, void *A, float *Z, void *amap,
               const void *Wq, const void *Wk, const void *Wv, const void *Wo_opt, void *Y,
               void *Y_extra_opt, void *ws, size_t ws_bytes, void *stream);

/*
 * A feed-forward core module for merged tokens (Sec. 4.2: the module between merge and unmerge may
 * be attention or an MLP; the ToMA_once variant of Sec. 5.1 merges once per block and runs every
 * module of the block on the merged tokens before one unmerge):
 *   Out = gelu(In W1) W2,   gelu(x) = x/2 (1 + erf(x / sqrt 2)),  no biases.
 * The paper does not fix the MLP's form; this is the plain two-layer GELU block.  A block in the
 * ToMA_once style is toma_merge / toma_merge_cached, toma_attend, toma_mlp, toma_unmerge.
 *   dtype   toma_dtype of every tensor
 *   In      in       [rows, C]       rows = all token rows of the batch, e.g. B * (D + t_extra)
 *   W1      in       [C, hidden]     row-major, y = x W
 *   W2      in       [hidden, C]
 *   Hbuf    scratch  [rows, hidden]  caller-owned, contents undefined afterwards
 *   Out     out      [rows, C]       may not alias In
 * Limits: C % 32 == 0 and hidden % 32 == 0.  Errors as for the other calls.
 */
int toma_mlp(int32_t dtype, int32_t rows, int32_t C, int32_t hidden, const void *In, const void *W1,
             const void *W2, void *Hbuf, void *Out, void *stream);

/*
 * Profiling aid for benchmarks (not part of the method; for callers that want per-kernel times).
 * While enabled, every kernel the library launches is bracketed by two HIP events recorded on the
 * launch stream (this is the one place where the library creates HIP objects: events, kept in a
 * pool until the process ends).  toma_profile_read waits for the recorded events of all kernels,
 * then returns and clears the launch count and summed duration (ms) of the named kernel.
 * toma_profile_kernel_name(i) enumerates the names (NULL past the last).  Enabling or disabling
 * clears all totals.  Not meant to be enabled under HIP graph capture.  The three calls may come from
 * any thread; a launch in flight on another thread while totals are read or cleared is counted
 * whole, either before or after.
 */
int toma_profile_enable(int on);
const char *toma_profile_kernel_name(int i);
int toma_profile_read(const char *kernel, int32_t *launches, float *total_ms);
/* Block tile the merge (which = 0) or unmerge (which = 1) product of this descriptor runs with, or
 * (which = 2) the write pass of the two-pass merge weights (rows = sources, columns = destinations):
 * out3 = {rows of the output per workgroup, columns, K split}.  A benchmark that holds the block map
 * can count from it which K steps (128 bytes of elements each) a workgroup's tile runs and so the
 * products actually executed.  Host arithmetic only; TOMA_ERR_UNSUPPORTED when the product does not
 * take the tiled path. */
int toma_profile_map_product(const toma_desc *desc, int which, int32_t *out3);
/* toma_select (Sec. 4.1, Alg. 2) with the greedy kernel replaced by a variant of itself that also
 * adds up, per wave, the shader clocks spent in each part of a round - a measurement aid for the one
 * kernel whose time is a chain of dependent steps rather than bytes or products.  idx as toma_select.
 * parts: device, 8 words per (sample, region) and wave, [B * P][waves][8], waves = 8 for regions of
 * 256 tokens and 2 for regions of 64 (other region sizes: TOMA_ERR_UNSUPPORTED): sums over the
 * rounds of 0 keys read and argmax found, 1 row of the pick posted and first barrier, 2 own columns
 * read and the changed ones found, 3 changed columns applied and atomics issued, 4 second barrier
 * (with the wait for the busiest wave); 5 rounds; 6 changed columns this wave owned; 7 zero.
 * Reading the counter costs about 30 clocks per part. */
int toma_profile_greedy_parts(const toma_desc *desc, const void *X, int32_t *idx, uint64_t *parts, void *ws,
                              size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TOMA_H */
