/*
 * isa.h -- C ABI of the In-Context Sparse Attention (ISA) library for AMD MI355X (gfx950).
 *
 * ISA (the paper's Sec. 3 and Algorithms 1 and 2) replaces the softmax attention of an
 * in-context video-editing transformer, whose token sequence is a source segment followed
 * by one or more context references, by four stages:
 *   1. pre-selection: score context key/value blocks by pooled attention and keep a top-k;
 *   2. query grouping: split query blocks by the sharpness of their pooled attention row;
 *   3. exact attention of the sharp query blocks over the source + kept context keys;
 *   4. block-wise 0-th order Taylor attention of the remaining query blocks, in which a
 *      key/value block enters through its mean key, mean value and token count;
 * and writes every result at its token's original position.
 *
 * Conventions shared by all entry points
 *   - Every function returns ISA_OK (0) or a negative isa_status.  Nothing throws, aborts or
 *     prints.  isa_strerror() names a status.
 *   - `q`, `k`, `v`, `out`, `workspace` and every array argument described as "device" are
 *     device pointers owned by the caller.  `isa_problem` and the arrays it points to
 *     (`seg_ptr`, `seg_len`) are host memory, read during the call only.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and the call returns without synchronising.  The library allocates no memory (isa_attention_simple excepted,
 *     see there) and keeps no per-problem state between calls: everything a later call needs is in the caller's
 *     workspace.  Process-wide switches exist for tests and measurement only (isa_set_mfma,
 *     isa_time_attention_kernel, at the end of this file) and are not meant to be flipped while calls are in flight.
 *   - Tensors q, k, v, out are [B, H, S_max, D] with element strides stride_b, stride_h,
 *     stride_t and a contiguous last dimension.  Batch item b holds S_b = sum of its segment
 *     lengths tokens, source segment first; rows S_b .. S_max-1 are neither read nor written.
 *   - Blocks: every segment is cut into blocks of `block` tokens starting at the segment's
 *     first token, so the last block of a segment may be short.  Block indices run over the
 *     source blocks first (0 .. T_src-1), then the context blocks.  T_max is the largest
 *     per-batch block count; per-(batch, head) block arrays are laid out [B, H, T_max].
 *   - Supported shapes: D in {64, 128}; block in {64, 128}; 1 <= B <= ISA_MAX_BATCH; at most
 *     ISA_MAX_SEGMENTS segments over all batch items; at most ISA_MAX_BLOCKS blocks per batch
 *     item; strides multiples of 8 elements; token tensors and block-mean arrays 16-byte aligned (ISA_ERR_SHAPE
 *     otherwise); gamma finite.
 */
#ifndef ISA_H
#define ISA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ISA_MAX_BATCH 8
#define ISA_MAX_SEGMENTS 32
#define ISA_MAX_BLOCKS 4096
#define ISA_STATIC_SCRATCH_BYTES (128u << 20) /* device scratch held by the library itself, see isa_attention_static */

typedef enum {
  ISA_OK = 0,
  ISA_ERR_NULL = -1,        /* a required pointer is NULL */
  ISA_ERR_SHAPE = -2,       /* B, H, D, block, segments or strides outside the supported set */
  ISA_ERR_RATIO = -3,       /* a ratio outside [0, 1] or not finite */
  ISA_ERR_DTYPE = -4,       /* dtype is neither ISA_BF16 nor ISA_F32 */
  ISA_ERR_UNSUPPORTED = -5, /* a non-finite gamma; a bf16, D = 128, block = 128 problem whose tokens of one (batch, head)
                               span 4 GiB or more (S_max * stride_t * 2 bytes: the matrix-core kernels use 32-bit byte
                               offsets; isa_set_mfma(0) selects the portable kernels, which have no such limit); a call
                               that is not available in the stream's state (isa_attention_simple under capture) */
  ISA_ERR_WORKSPACE = -6,   /* workspace NULL, misaligned (256 B) or smaller than required */
  ISA_ERR_HIP = -7          /* a HIP runtime call or kernel launch failed */
} isa_status;

typedef enum { ISA_BF16 = 0, ISA_F32 = 1 } isa_dtype;

/* The problem statement of Algorithm 1: shapes, segments and the three ratios. */
typedef struct isa_problem {
  int32_t B, H, D;
  int32_t dtype;          /* isa_dtype of q, k, v and out.  bf16 is the production path; fp32 is the checking mode */
  int32_t block;          /* tokens per query block and per key/value block (the paper's b = L_Q = L_K) */
  const int32_t* seg_ptr; /* host [B+1]: batch item b owns seg_len[seg_ptr[b] .. seg_ptr[b+1]) */
  const int32_t* seg_len; /* host: first segment of a batch item = source, the others = context references */
  int64_t stride_b, stride_h, stride_t; /* element strides of q, k, v and out */
  double keep_ratio;      /* Select Ratio alpha_s: fraction of context blocks kept (Sec. 3, Eq. 1-2) */
  double full_frac;       /* fraction of query blocks given exact attention (Alg. 1 Stage 3) */
  double exact_frac;      /* No-Sparsity Ratio alpha_ns: fraction of kept blocks a Taylor query block still
                             evaluates exactly (Alg. 2 Stage 2) */
  double gamma;           /* coarse stacking factor of Alg. 1 (Stage 5): out += gamma * O_coarse; 0 = no residual */
} isa_problem;

/* Block and list counts of one batch item, all derived on the host in double precision. */
typedef struct isa_counts {
  int32_t S;       /* tokens */
  int32_t T;       /* blocks */
  int32_t T_src;   /* source blocks */
  int32_t T_ctx;   /* context blocks */
  int32_t k_keep;  /* floor(keep_ratio * T_ctx) kept context blocks */
  int32_t T_new;   /* T_src + k_keep: length of kv_list */
  int32_t n_flat;  /* floor((1 - full_frac) * T): query blocks of the Taylor branch */
  int32_t n_full;  /* T - n_flat: query blocks of the exact branch */
  int32_t k_exact; /* floor(exact_frac * T_new): exact blocks per Taylor query block */
  int32_t T_max;   /* largest T over the batch (stride of block arrays) */
} isa_counts;

/* Host only.  Validates `p` and reports the counts of batch item `b`.  Needs no GPU. */
int isa_get_counts(const isa_problem* p, int b, isa_counts* out);

/* Host only.  Bytes of device workspace any entry point below needs for `p` (0 if `p` is invalid).
 * The workspace must be 256-byte aligned.  Its contents are scratch: undefined before and after. */
size_t isa_workspace_bytes(const isa_problem* p);

/* Where isa_attention leaves its intermediate results inside the workspace: byte offsets from the workspace pointer.
 * They let a caller (a test, a profiler, a model that logs sparsity patterns) read the block means, scores and index
 * lists the call actually used instead of recomputing them with the staged entry points.  Arrays that the problem does
 * not need are reported as ISA_NO_ARRAY. */
#define ISA_NO_ARRAY ((size_t)-1)
typedef struct isa_ws_layout {
  size_t bytes;                          /* = isa_workspace_bytes(p) */
  size_t qc, kc, vc;                     /* fp32 [B, H, T_max, D]: block means (Alg. 1 Stage 1) */
  size_t s_ctx, sharp;                   /* fp32 [B, H, T_max]: Eq. 1 saliency of the context blocks; sharpness (Stage 3) */
  size_t kv_list, full_list, flat_list;  /* int32 [B, H, T_max], as isa_select writes them */
  size_t exact_mask;                     /* uint32 [B, H, T_max, ceil(T_max/32)]; only when exact_frac > 0 */
  size_t o_coarse;                       /* fp32 [B, H, T_max, D]; only when gamma != 0 */
  size_t nlse;                           /* fp32 [B, H, S_max]: minus the base-2 log-sum-exp of every query row's scaled
                                            logits, as isa_attention_backward wants it (Taylor rows: with the n_j weights
                                            of Eq. 4, and, when exact_frac == 0, of the logits against the mean keys minus
                                            the mean key of block 0, which is what the kernels multiply); only for bf16,
                                            D = 128, block = 128 */
} isa_ws_layout;

/* Host only.  Fills `out` for `p`; the layout is a function of the problem alone.  Needs no GPU. */
int isa_workspace_layout(const isa_problem* p, isa_ws_layout* out);

/* Algorithm 1, all stages, for every (batch, head): out = ISA(q, k, v).
 * With gamma != 0 the coarse residual of Stage 5 is added: every token of query block i receives
 * gamma * O_coarse[i], where O_coarse = S_coarse vc (Stage 1; O_coarse has one row per block, so a block's row is
 * shared by its tokens).  `out` is written for every real token.  Errors: see isa_status. */
int isa_attention(const isa_problem* p, const void* q, const void* k, const void* v, void* out,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* Standard attention softmax(q k^T / sqrt(D)) v (Sec. 2 "Standard Attention") over all S_b keys of
 * each batch item; the ratios in `p` are ignored.  This is the kernel ISA is timed against. */
int isa_dense_attention(const isa_problem* p, const void* q, const void* k, const void* v, void* out,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* Convenience form: B = 1, bf16, contiguous [H, n_src + n_ctx, D] tensors, one context segment,
 * exact_frac = 0.  Unlike every other entry point it obtains its workspace with hipMallocAsync on
 * `hip_stream` and releases it with hipFreeAsync, so it is not for callers that must not allocate (isa_attention_static
 * is), and it returns ISA_ERR_UNSUPPORTED when `hip_stream` is being captured into a graph. */
int isa_attention_simple(const void* q, const void* k, const void* v, int H, int D, int n_src, int n_ctx,
                         double keep_ratio, double full_frac, int block, void* out, void* hip_stream);

/* isa_attention for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same result as
 * isa_attention, but the scratch memory is a fixed array of ISA_STATIC_SCRATCH_BYTES inside the library's own device
 * image (every GPU the library runs on holds one copy until the process ends); the call allocates and frees nothing.
 * Limits: the forward-only workspace of `p` (the arrays isa_attention needs, without those it would leave for
 * isa_attention_backward) must fit that array, else ISA_ERR_WORKSPACE and nothing is launched; at D = 128 in bf16 that is
 * about 330 000 head-tokens (H * S), e.g. 40 heads of 8 000 tokens.  No backward call can follow it.  The array is shared
 * by every call on the same GPU and keeps the previous call's contents (no call relies on them): two calls that overlap on
 * one GPU (different streams, different threads) race; calls on one stream are ordered.  The first call on a device
 * looks the array's address up (hipGetSymbolAddress), so make it before a stream capture begins. */
int isa_attention_static(const isa_problem* p, const void* q, const void* k, const void* v, void* out, void* hip_stream);

/* ---- staged entry points: one per stage, so each can be checked on its own ---------------- */

/* Alg. 1 Stage 1 / Alg. 2 Stage 1: block means over each block's real tokens.
 * qc, kc, vc: device fp32 [B, H, T_max, D]; rows past a batch item's T are not written. */
int isa_block_means(const isa_problem* p, const void* q, const void* k, const void* v,
                    float* qc, float* kc, float* vc, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Pooling attention (Sec. 2) + Eq. 1 + the sharpness of Alg. 1 Stage 3.
 * S_coarse = row softmax over all T key blocks of qc kc^T / sqrt(D).
 * s_ctx: device fp32 [B, H, T_max]; entry j < T_ctx = mean over source query blocks of S_coarse[i, T_src + j].
 * sharp: device fp32 [B, H, T_max]; entry i < T = population variance of S_coarse[i, 0..T_src).
 * z: device fp32 [B, H, T_max, T_max] or NULL; if given, receives the scaled logits qc kc^T / sqrt(D). */
int isa_coarse_scores(const isa_problem* p, const float* qc, const float* kc, float* s_ctx, float* sharp, float* z,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* The pooled attention output of Alg. 1 Stage 1: O_coarse = S_coarse vc, with S_coarse as in isa_coarse_scores.
 * o_coarse: device fp32 [B, H, T_max, D]; rows past a batch item's T are not written. */
int isa_coarse_output(const isa_problem* p, const float* qc, const float* kc, const float* vc, float* o_coarse,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/* Eq. 2 selection and the Alg. 1 Stage 3 split, as integer work on given fp32 scores.
 * Rankings are by descending score, ties to the lower index; all lists are stored ascending.
 * kv_list:   device int32 [B, H, T_max]; first T_new entries = source blocks 0..T_src-1, then kept context blocks.
 * full_list: device int32 [B, H, T_max]; first n_full entries = query blocks of the exact branch.
 * flat_list: device int32 [B, H, T_max]; first n_flat entries = query blocks of the Taylor branch.
 * Entries past those counts are set to -1.
 * z / exact_mask: only read / written when exact_frac > 0 (both may be NULL otherwise).
 * exact_mask: device uint32 [B, H, T_max, ceil(T_max/32)]; in the row of the Taylor query block stored at position r
 * of flat_list, bit (t mod 32) of word t/32 is set iff kv_list[t] is one of its k_exact exact blocks (largest z,
 * ties to the lower position in kv_list; Alg. 2 Stage 2). */
int isa_select(const isa_problem* p, const float* s_ctx, const float* sharp, const float* z,
               int32_t* kv_list, int32_t* full_list, int32_t* flat_list, uint32_t* exact_mask,
               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Alg. 1 Stages 4-5 on given lists: exact attention (online softmax, Alg. 2 Part A) for the blocks of
 * full_list, block-wise 0-th order Taylor attention (Eq. 3-4, Alg. 2 Parts A+B, with a block's real token
 * count in place of L_K) for the blocks of flat_list, both over the blocks of kv_list, each result stored at its
 * token's position in `out`.  kc, vc: block means as written by isa_block_means.  exact_mask may be NULL when
 * exact_frac == 0.  o_coarse: as written by isa_coarse_output; read only when gamma != 0 (then required), in which
 * case gamma * o_coarse[block] is added to every token of the block (Stage 5).  The lists must be valid (in range,
 * no duplicates); they are not checked: an entry out of range is forced into range (a wrong result, no access outside
 * the tensors). */
int isa_attend(const isa_problem* p, const void* q, const void* k, const void* v, const float* kc, const float* vc,
               const int32_t* kv_list, const int32_t* full_list, const int32_t* flat_list, const uint32_t* exact_mask,
               const float* o_coarse, void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Backward pass of isa_attention / isa_attend (the paper states that the operator is trainable and gives no
 * formulas, Sec. 4 "Implementation Detail and Analysis"): the gradient of Alg. 1 Stages 4-5 with respect to q, k and v
 * with every index decision of Stages 2-3 held fixed (kept blocks, query groups: piecewise constant in the inputs),
 * including the gradient through the block means of the Taylor branch (Eq. 4: a mean key's gradient is spread evenly
 * over its block's tokens).
 * q, k, v, out: as given to / written by the forward call; d_out: gradient of the loss with respect to `out`;
 * dq, dk, dv: receive the gradients.  All seven are device bf16 tensors with the layout and strides of the problem;
 * every row of dq, dk and dv is written (with gamma == 0, keys and values of context blocks that were not kept get
 * zeros).
 * kv_list, full_list, flat_list, exact_mask: the device lists (and, when exact_frac > 0, the exact-set bits, as written
 * by isa_select) the forward call ran with, or all NULL for those that isa_attention left in the workspace.
 * The workspace must be the one the forward call used, untouched since: it holds the log-sum-exp of every query row and
 * the part of every output element that its rounding to bf16 cut off (so that rowsum(d_out * out) is taken from the
 * unrounded result) (and, when the lists are taken from it, the block table, the block means and O_coarse, which are then not computed again).
 * With gamma != 0 the gradient of the coarse residual (through the means of all blocks, query blocks included) is part
 * of the result.
 * Only for bf16, D = 128, block = 128 with the MFMA kernels selected (ISA_ERR_UNSUPPORTED otherwise).  The library keeps
 * no record of the forward call, so it cannot check the following and the gradients are undefined (no access outside the
 * tensors and the workspace) if it does not hold: the forward call ran the MFMA kernels (isa_set_mfma was 1), was
 * isa_attention when the lists are NULL here, and nothing else has used the workspace since.  Asynchronous on hip_stream; fp32
 * accumulation, no atomics: results are reproducible run to run. */
int isa_attention_backward(const isa_problem* p, const void* q, const void* k, const void* v, const void* out,
                           const void* d_out, const int32_t* kv_list, const int32_t* full_list,
                           const int32_t* flat_list, const uint32_t* exact_mask, void* dq, void* dk, void* dv,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- prologue: tile-order flattening and decoupled rotary embedding ------------------------ */

/* Where the tokens of every segment sit and how they are to be embedded.
 * The paper fixes that tokens are grouped into contiguous spatiotemporal tiles which are flattened in tile order before
 * the sequence is cut into blocks (Sec. 2 "Block Sparse Attention"), and that the rotary embedding is applied to the
 * source and to the context independently with the positions of each reset to zero (Sec. 4, third design choice of the
 * editing model); tile shape and embedding layout are parameters here. */
typedef struct isa_grid {
  const int32_t* seg_grid; /* host [number of segments of the problem][3]: (t, h, w) of each segment, in the order of
                              seg_len; t * h * w must equal the segment's length */
  int32_t tile[3];         /* (tt, th, tw) >= 1: tile shape.  Tiles are enumerated row-major over tile coordinates
                              (w fastest), tokens row-major inside a tile; tiles at the far edges of a grid that the shape
                              does not divide are clipped */
  int32_t rope_dims[3];    /* channels turned by the t, h and w coordinate: each even and >= 0, sum <= D; they occupy
                              the head dimension in this order from channel 0, channels past the sum pass through */
  double rope_theta;       /* base > 0: pair j (channels 2j, 2j+1) of an axis with d channels turns counter-clockwise by
                              coordinate * rope_theta^(-2j/d) radians */
} isa_grid;

/* One streaming pass that prepares the operator's inputs.  q_in, k_in, v_in: device tensors of the problem's dtype,
 * layout and strides whose segments are row-major over their grids (w fastest).  q_out, k_out, v_out (same layout and
 * strides, distinct from the inputs): position p of a segment receives the p-th token of its tile order; q and k
 * rotated by their grid coordinates counted from zero inside the segment, v unchanged.  qc, kc, vc: all NULL, or
 * device fp32 [B, H, T_max, D] that receive the block means of the three outputs (of the stored, i.e. rounded, values),
 * as isa_block_means would compute them from q_out, k_out, v_out: the first stage of Alg. 1 fused into the same pass.
 * The ratios of `p` are not used.  Pointers must be 16-byte aligned.  No workspace; asynchronous on hip_stream.
 * Errors: ISA_ERR_NULL; ISA_ERR_SHAPE for a grid that does not match its segment, a bad tile or rope_dims,
 * a misaligned or aliased pointer; ISA_ERR_UNSUPPORTED for a non-positive or non-finite rope_theta. */
int isa_prologue(const isa_problem* p, const isa_grid* grid, const void* q_in, const void* k_in, const void* v_in,
                 void* q_out, void* k_out, void* v_out, float* qc, float* kc, float* vc, void* hip_stream);

/* Backward pass of isa_prologue: the prologue is linear (a rotation of every channel pair of q and k, then a reordering of
 * the tokens), so the gradient with respect to its inputs is its transpose applied to the gradient with respect to its
 * outputs: row p of a segment's tile order goes back to its row-major place, and every pair of dq and dk turns the other
 * way.  dq_out, dk_out, dv_out: gradients with respect to q_out, k_out, v_out (what isa_attention_backward returns when
 * the operator ran on the prologue's outputs); dq_in, dk_in, dv_in receive the gradients with respect to q_in, k_in, v_in.
 * Same dtype, layout, strides, alignment and aliasing rules as isa_prologue.  The fused block means need no term of their
 * own: isa_attention_backward already returns the gradient through the means as part of dq, dk, dv. */
int isa_prologue_backward(const isa_problem* p, const isa_grid* grid, const void* dq_out, const void* dk_out,
                          const void* dv_out, void* dq_in, void* dk_in, void* dv_in, void* hip_stream);

/* The inverse reordering for one tensor (the operator's output on its way back to the model): x_tiled in tile order ->
 * x_raster row-major per segment; same dtype, layout and strides, distinct buffers.  rope_dims and rope_theta are not
 * used. */
int isa_untile(const isa_problem* p, const isa_grid* grid, const void* x_tiled, void* x_raster, void* hip_stream);

/* Name of a status code; never NULL. */
const char* isa_strerror(int status);

/* hipError_t (as int) of the most recent failing HIP call made by this library on the calling thread,
 * 0 if none.  Only meaningful right after a call returned ISA_ERR_HIP. */
int isa_last_hip_error(void);

/* Selects the attention kernels used for bf16 problems with D = 128 and block = 128:
 * 1 (default) = MFMA kernels, 0 = the portable scalar kernels that also serve fp32 and the other shapes.
 * Returns the previous setting.  Process-wide; meant for tests and comparisons. */
int isa_set_mfma(int enabled);

/* Measurement hook.  isa_time_attention_kernel(1) makes every later launch of the MFMA attention kernel record a
 * pair of HIP events (created by the library on first use) just before and just after the kernel on the launch
 * stream; isa_time_attention_kernel(0) switches that off.  isa_last_attention_kernel_ms() waits for the most
 * recently recorded pair and returns the kernel's duration in milliseconds (ISA_ERR_UNSUPPORTED if none was
 * recorded).  Process-wide; not for concurrent callers. */
int isa_time_attention_kernel(int enabled);
int isa_last_attention_kernel_ms(float* ms);

#ifdef __cplusplus
}
#endif
#endif /* ISA_H */
