/*
 * rainfusion.h -- C ABI of the MI355X (gfx950) implementation of RainFusion's
 * per-head sparse 3D attention (arxiv 2505.21036): the ARM head classifier
 * (Sec. 3.3, Eq. 6, Alg. 1) and the block-sparse attention forward pass that
 * applies each head's pattern (Sec. 3.1-3.2, Eq. 1-5; Fig. 2a).
 *
 * Conventions for every entry point
 *   - Tensors are DEVICE pointers owned by the caller: bf16, contiguous
 *     [B, nH, N, D] (batch, head, token, channel), 16-byte aligned (the kernels move 16
 *     bytes at a time; RF_ERR_ALIGN otherwise).  The library neither frees nor keeps
 *     them.  D is 64, 96 or 128.
 *   - Token order (Sec. 3.1): T frames of H*W tokens each, frame-major, row-major
 *     inside a frame; text_len text tokens follow the video tokens, or precede
 *     them under RF_FLAG_TEXT_FIRST.  N = T*H*W + text_len.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and never synchronise it, except that the first call for a new
 *     (layout, params, block) builds and uploads its block lists synchronously.  After
 *     such a warm-up call a sequence of calls only launches kernels (no memsets, no
 *     allocations) and can be captured into a HIP graph; the ARM's results are bitwise the
 *     same from call to call, the attention's under RF_FLAG_FIXED_ORDER.  All per-call device state lives in the caller's workspaces, so
 *     any number of calls may be in flight as long as each has its own workspace.  The
 *     library keeps at most 16 block lists per process (least recently used first out;
 *     making room synchronises the device).
 *   - Return value: RF_OK or a negative rf_status.  Arguments are validated before
 *     any GPU work, so a bad argument never launches a kernel.
 *   - `params == NULL` selects the paper's defaults (Sec. 4.1: both bandwidths 1/4,
 *     checkerboard stride 2) and sampling interval T.
 */
#ifndef RAINFUSION_H
#define RAINFUSION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Latent video shape (Sec. 3.1) plus the number of appended text tokens. */
typedef struct {
    int32_t T, H, W, text_len;
} rf_layout;

/* Pattern parameters.
 *   bw_spatial  : Spatial head (Eq. 3) keeps frames f' with |f - f'| <= floor(bw_spatial * T).
 *   bw_temporal : Temporal head keeps in-frame positions p' with |p - p'| <= floor(bw_temporal * H*W),
 *                 in every frame.  Both products are formed in double precision.
 *   tex_stride  : tau of Eq. 4; a key at row y, column x of any frame survives iff (y - x) mod tau == 0.
 *   sample_interval : omega of Sec. 3.3 (global sampling keeps tokens 0, omega, 2*omega, ...); 0 means T.
 *   flags       : 0 or an OR of RF_FLAG_* below.
 * Text tokens attend and are attended densely under every pattern and are never sampled by the ARM. */
typedef struct {
    float bw_spatial, bw_temporal;
    int32_t tex_stride;
    int32_t sample_interval;
    int32_t flags; /* RF_FLAG_* */
} rf_params;

/* Two-head ablation (Sec. 4.2, Tab. 2 rows without "Te"): the ARM sends a head that matches neither
 * the Temporal nor the Spatial mask to RF_DENSE instead of RF_TEXTURAL. */
#define RF_FLAG_TWO_HEAD 1
/* The text tokens are the FIRST text_len rows of every tensor and the video tokens follow them (the
 * order of models that prepend the prompt).  The paper does not place the text tokens; the masks
 * are defined on the video tokens' (frame, row, column), so only where those sit changes. */
#define RF_FLAG_TEXT_FIRST 2
/* rf_sparse_attention treats every head as RF_DENSE and does not read head_class (which may then be
 * NULL): the "first 10 % of the timesteps dense" policy of Sec. 4.1 without touching the class
 * buffer.  Ignored by the ARM. */
#define RF_FLAG_FORCE_DENSE 4
/* rf_sparse_attention visits each query block's key tiles in an order fixed by the layout alone, which
 * makes O bitwise identical from call to call.  Without the flag a query block starts its (cyclic) walk
 * over its tiles wherever the workgroups already running on the same part of the GPU are, so that they
 * share K/V tiles through the L2 cache: every tile is still visited exactly once, but the fp32 sums are
 * formed in an order that depends on timing, so the last bit of O can differ between calls (faster,
 * chiefly on Spatial and Temporal heads).  Ignored by the ARM, whose results are always reproducible. */
#define RF_FLAG_FIXED_ORDER 8
/* rf_sparse_attention runs the variant of its kernel in which a wavefront owns 64 query rows instead
 * of 32 (half the shared-memory operand reads per matrix instruction, one wavefront per SIMD, the
 * softmax of one tile interleaved with the matrix instructions of its neighbours).  Same result to
 * rounding order.  Only with head_dim 128 and block 256 (RF_ERR_PARAM otherwise).  Ignored by the ARM. */
#define RF_FLAG_WIDE_ROWS 16

#define RF_MAX_BANDWIDTHS 4 /* candidate bandwidths of the per-head bandwidth variant */

enum rf_head_class { RF_SPATIAL = 0, RF_TEMPORAL = 1, RF_TEXTURAL = 2, RF_DENSE = 3 };
enum rf_sample_mode { RF_SAMPLE_FIRST_FRAME = 0, RF_SAMPLE_EQUAL_INTERVAL = 1 };
enum rf_status {
    RF_OK = 0,
    RF_ERR_NULL = -1,      /* a required pointer is NULL */
    RF_ERR_SHAPE = -2,     /* B, nH < 1, D not in {64, 96, 128}, or sizes overflow int32 token indices */
    RF_ERR_LAYOUT = -3,    /* T, H, W < 1 or text_len < 0 */
    RF_ERR_PARAM = -4,     /* bandwidth outside [0, 1], tex_stride < 1, sample_interval < 0, unknown flags, bad sample_mode,
                              threshold not in [0, 1] or NaN */
    RF_ERR_BLOCK = -5,     /* block not 64, 128, 256 or 384 */
    RF_ERR_WORKSPACE = -6, /* a required workspace is NULL, or a workspace is too small or misaligned */
    RF_ERR_HIP = -7,       /* a HIP runtime call failed (allocation, copy or launch) */
    RF_ERR_ALIGN = -8      /* a tensor is not 16-byte aligned, or the attention workspace not 256-byte aligned */
};

/*
 * ARM, Alg. 1: classify every head of one attention layer.
 *   For each (b, h): R_hat = recall (Eq. 6) of the Temporal mask on the sampled Q', K'
 *   (first-frame tokens in RF_SAMPLE_FIRST_FRAME mode, equal-interval tokens in
 *   RF_SAMPLE_EQUAL_INTERVAL mode); R_tilde = recall of the Spatial mask on the
 *   equal-interval sample.  Recall is the mean over sampled query rows of the softmax
 *   mass (scores Q'K'^T / sqrt(D)) that falls on keys the mask keeps.
 *   head_class = TEMPORAL if R_hat >= threshold, else SPATIAL if R_tilde >= threshold,
 *   else TEXTURAL (RF_DENSE under RF_FLAG_TWO_HEAD).
 * Q, K        : device, bf16 [B, nH, N, D].
 * head_class  : device, int32 [B*nH], written.
 * recalls     : device, float [B*nH*2] = {R_hat, R_tilde} per head, written; may be NULL.
 * workspace   : device scratch of at least rf_arm_workspace_bytes() bytes (per-row recalls;
 *               contents undefined afterwards); two calls that overlap in time need two workspaces.
 * The per-row recalls are reduced in a fixed order, so results are run-to-run identical.
 */
int rf_arm_classify(const void *Q, const void *K, int B, int nH, int D, const rf_layout *layout,
                    const rf_params *params, int sample_mode, float threshold, int32_t *head_class,
                    float *recalls, void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of device scratch rf_arm_classify needs for this problem; 0 if the arguments are invalid. */
size_t rf_arm_workspace_bytes(int B, int nH, const rf_layout *layout, const rf_params *params);

/*
 * rf_arm_classify for callers that cannot allocate device memory or pass a workspace along (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments
 * minus the workspace, same kernels, same results.  The per-row recalls go to a static array of
 * RF_ARM_STATIC_SCRATCH_BYTES inside the library's device image instead (every GPU the library
 * runs on holds one until the process ends).  The call allocates and frees nothing.
 *   - Problems that need more scratch than that (rf_arm_workspace_bytes() > RF_ARM_STATIC_SCRATCH_BYTES)
 *     are refused with RF_ERR_WORKSPACE before any GPU work.
 *   - All calls on one GPU share the array: calls that overlap in time on one GPU (different
 *     streams, or replays of graphs that captured it) race with each other.  Nothing in it has to
 *     start at zero; its contents are undefined afterwards.
 */
#define RF_ARM_STATIC_SCRATCH_BYTES (2u << 20)
int rf_arm_classify_noalloc(const void *Q, const void *K, int B, int nH, int D, const rf_layout *layout,
                            const rf_params *params, int sample_mode, float threshold, int32_t *head_class,
                            float *recalls, void *stream);

/*
 * RainFusion+ (Sec. 4.3): ARM with per-head bandwidth.  Alg. 1's two recalls are measured once
 * per candidate bandwidth (bandwidths[k] replaces both bw_temporal and bw_spatial of `params`),
 * in the same pass over the sampled scores.  A head is TEMPORAL with the narrowest candidate
 * whose R_hat >= threshold if there is one, else SPATIAL with the narrowest candidate whose
 * R_tilde >= threshold, else TEXTURAL (the paper uses candidates 0.5, 0.25, 0.125 and 90 %).
 * bandwidths  : HOST, float [n_bw], each in [0, 1], 1 <= n_bw <= RF_MAX_BANDWIDTHS, any order.
 * head_class  : device, int32 [B*nH], written.
 * head_bw     : device, int32 [B*nH], written: index into bandwidths, -1 for TEXTURAL heads.
 * recalls     : device, float [B*nH][2][n_bw] = R_hat per candidate, then R_tilde per candidate; may be NULL.
 * workspace   : device scratch of at least n_bw * rf_arm_workspace_bytes() bytes.
 * Everything else as rf_arm_classify.
 */
int rf_arm_classify_plus(const void *Q, const void *K, int B, int nH, int D, const rf_layout *layout,
                         const rf_params *params, int sample_mode, float threshold, const float *bandwidths,
                         int n_bw, int32_t *head_class, int32_t *head_bw, float *recalls, void *workspace,
                         size_t workspace_bytes, void *stream);

/*
 * Sparse attention forward, Eq. 1-2 with the mask of each head's pattern (Eq. 3-5):
 *   O[b,h,i,:] = sum_j softmax_j(q_i . k_j / sqrt(D) over kept j) * v_j.
 * The mask is token-level; `block` (64, 128, 256 or 384) is the number of query rows per block (= per
 * workgroup: larger blocks share each K/V tile among more queries and run faster on long sequences), and
 * (query block, 64-key tile) pairs with no kept token pair are skipped, so O does not
 * depend on it.  Scores and sums are accumulated in fp32, O is rounded to bf16.
 * Q, K, V     : device, bf16 [B, nH, N, D].
 * head_class  : device, int32 [B*nH], values of rf_head_class; read on the device, so the
 *               output of rf_arm_classify can be passed on without a host round trip.
 *               Values outside 0..3 are treated as RF_DENSE.  May be NULL under RF_FLAG_FORCE_DENSE.
 * O           : device, bf16 [B, nH, N, D], written.
 * workspace   : device scratch, 256-byte aligned, REQUIRED: at least RF_ATTENTION_MIN_WORKSPACE bytes
 *               (the kernel's work-queue counters, zeroed by the call itself).  If it has
 *               rf_attention_workspace_bytes() bytes or more, K and V of the heads that profit are
 *               first copied into the rest of it in a friendlier order: the kept keys of Textural heads
 *               made contiguous (K_C, V_C of Eq. 5), the tokens of Temporal heads in position-major order
 *               (same in-frame position of all frames adjacent), where the Temporal band is one
 *               contiguous run of keys per query block.  The result is the same either way.  Contents
 *               undefined afterwards; calls that overlap in time need separate workspaces.
 */
#define RF_ATTENTION_MIN_WORKSPACE 512
int rf_sparse_attention(const void *Q, const void *K, const void *V, const int32_t *head_class, int B,
                        int nH, int D, const rf_layout *layout, const rf_params *params, int block,
                        void *O, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Sparse attention with per-head bandwidth (the attention half of RainFusion+): as
 * rf_sparse_attention, but head (b, h) uses bandwidths[head_bw[b*nH + h]] for its Spatial or
 * Temporal band instead of params' (TEXTURAL and DENSE heads, and indices outside 0..n_bw-1,
 * ignore it / fall back to bandwidths[0]).
 * head_bw     : device, int32 [B*nH].   bandwidths : HOST, float [n_bw], 1 <= n_bw <= RF_MAX_BANDWIDTHS.
 */
int rf_sparse_attention_plus(const void *Q, const void *K, const void *V, const int32_t *head_class,
                             const int32_t *head_bw, const float *bandwidths, int n_bw, int B, int nH, int D,
                             const rf_layout *layout, const rf_params *params, int block, void *O,
                             void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of the full workspace of rf_sparse_attention (the counters plus room for a copy of K and V);
 * 0 if the arguments are invalid. */
size_t rf_attention_workspace_bytes(int B, int nH, int D, const rf_layout *layout, const rf_params *params);

/*
 * Host-side view of the list rf_sparse_attention walks (Fig. 2a "applying the sparse
 * pattern"): for pattern `cls`, which key tiles each query block visits.  Query blocks are
 * `block` rows; key tiles are always RF_KEY_TILE = 64 keys, so a list is never coarser than
 * a block x block tiling would be.  Pure host code, no GPU needed.
 *   row_ptr : host, int32 [nQB + 1] (nQB = ceil(N / block)), written; may be NULL to only size.
 *   cols    : host, int32 [cap]; entry = key-tile index, plus RF_PLAN_PARTIAL if the pair
 *             contains a dropped token pair or runs past the last token (the kernel applies the
 *             token predicate there).  For RF_TEXTURAL, query blocks made only of video tokens
 *             index tiles of the COMPACTED key sequence (kept keys in token order, then text).
 *             cls = RF_LIST_TEMPORAL_POSITION_MAJOR gives the list a Temporal head walks when a
 *             workspace is given: query blocks and key tiles are then runs of the position-major
 *             order (see rf_plan_position_major).
 *   needed  : host, receives the number of entries.
 * Under RF_FLAG_TEXT_FIRST rows are counted in the order the kernel walks: video tokens first
 * (row r < T*H*W is token text_len + r), then the text tokens.
 * Returns RF_ERR_WORKSPACE if cap < *needed (nothing but *needed and row_ptr is written then).
 */
#define RF_PLAN_PARTIAL 0x40000000
#define RF_KEY_TILE 64
#define RF_LIST_TEMPORAL_POSITION_MAJOR 4
int rf_plan_host(const rf_layout *layout, const rf_params *params, int block, int cls,
                 int32_t *row_ptr, int32_t *cols, size_t cap, size_t *needed);

/*
 * Host-side view of how rf_sparse_attention schedules a head's query blocks under pattern `cls`
 * (scheduling only: it affects cache behaviour and load balance, never the result).
 *   order       : host, int32 [nQB], receives a permutation of 0..nQB-1.  First the blocks that hold
 *                 text rows (the long ones: text queries see every key): they are handed out, for all
 *                 heads, before anything else.  Then the other nV blocks in a locality order (token
 *                 order for RF_DENSE), of which XCD x of the GPU owns entries
 *                 [x * ceil(nV/8), (x+1) * ceil(nV/8)), head after head.
 *   first_entry : host, int32 [nQB] or NULL: per query block, the entry of its rf_plan_host list at
 *                 which its walk starts (it wraps around), chosen so that blocks in flight together
 *                 on an XCD sweep the same key tiles at the same time; 0 where the list is not one
 *                 sliding range of tiles.
 */
int rf_plan_order(const rf_layout *layout, const rf_params *params, int block, int cls, int32_t *order,
                  int32_t *first_entry);

/* Position-major order of the tokens: token_of (host, int32 [N]) receives, for every row of that
 * order, the token (row of the caller's tensors) it holds: video token (frame f, in-frame position
 * p) is row p*T + f, the text tokens are the last text_len rows.  Only RF_FLAG_TEXT_FIRST of
 * `params` (may be NULL) matters. */
int rf_plan_position_major(const rf_layout *layout, const rf_params *params, int32_t *token_of);

/* Drop every cached block list and free its device memory (synchronises the device). */
int rf_plan_clear(void);

/* Human-readable name of a status code. Never NULL. */
const char *rf_status_string(int status);

/* Library version, major*100 + minor. */
int rf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RAINFUSION_H */
