/*
 * varlen_attn.h -- C ABI of the packed variable-length causal attention library
 * for AMD MI355X (gfx950).
 *
 * The operation: a padding-free packed token stream [R rows, T tokens per row]
 * carries position ids that run 0..L-1 inside each example and restart at 0
 * (paper, Section 3 and Section 3.1).  The restart marks the example boundary.
 * From the ids the library derives cu_seqlens (Section 3, last paragraph) and
 * runs causal softmax attention, forward and backward, in which a token
 * attends only to earlier tokens of its own example ("correct cross-attention",
 * Table 1).  Rows are separate batch elements: token 0 of a row always starts
 * an example.
 *
 * Conventions
 *   - Unless marked "host", every pointer is DEVICE memory owned by the caller.
 *     The library allocates nothing, frees nothing and never synchronises; all
 *     work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).
 *   - Arguments are validated on the host before anything is launched; a
 *     non-zero status means nothing was enqueued (VA_ERR_HIP excepted).
 *   - Tensors are contiguous, token-major:
 *         Q, O, dO, dQ : [N, Hq,  d]      N = R * T
 *         K, V, dK, dV : [N, Hkv, d]
 *         LSE          : [Hq, N] float
 *     Query head h reads KV head h / (Hq / Hkv); Hq % Hkv == 0 is required.
 *   - Outputs are fully overwritten; inputs are never modified.
 *   - One va_pack_to_cu_seqlens call serves any number of forward / backward
 *     calls on the same packed stream (every layer of a model shares it).
 */
#ifndef VARLEN_ATTN_H
#define VARLEN_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  VA_OK = 0,
  VA_ERR_NULL = 1,        /* a required pointer is NULL                                    */
  VA_ERR_SHAPE = 2,       /* rows/tokens/heads/head_dim <= 0, N >= 2^31, Hq % Hkv != 0      */
  VA_ERR_UNSUPPORTED = 3, /* unknown dtype / id type / gradient type, head_dim > 256, Hq > 65535, or
                             (MFMA path) (tokens_per_row + 256) * Hq * d * 2 >= 2^32 - 256   */
  VA_ERR_WORKSPACE = 4,   /* plan buffer or workspace smaller than the *_bytes() query says */
  VA_ERR_HIP = 5          /* a launch failed (hipGetLastError after the launch)             */
} va_status;

typedef enum { VA_F32 = 0, VA_BF16 = 1, VA_F16 = 2 } va_dtype; /* element type of Q/K/V/O/dO and of the gradients */
typedef enum { VA_I32 = 0, VA_I64 = 1 } va_itype;   /* element type of position_ids                     */

/* The tile schedule is expressed in tiles of this many consecutive tokens of a packed row. */
#define VA_TILE 256
/* Tile index of a q_tile_order / kv_tile_order entry. */
#define VA_ORDER_TILE(entry) ((entry) & 0xffffff)

/*
 * Example boundaries and tile schedule of one packed stream.  A host struct of
 * device pointers into the caller's plan buffer; filled by va_segments_bind,
 * whose contents are written by va_pack_to_cu_seqlens.
 */
typedef struct va_segments {
  int32_t *cu_seqlens;    /* [N+1] capacity; entries 0..n valid: start token of each example, cu[n] = N */
  int32_t *seg_id;        /* [N]  index of the example holding token t                                   */
  int32_t *seg_start;     /* [N]  first token of that example  (= cu[seg_id[t]])                         */
  int32_t *seg_end;       /* [N]  one past its last token      (= cu[seg_id[t] + 1])                     */
  int32_t *meta;          /* [8]  meta[0] = n (examples), meta[1] = max_seqlen; rest reserved            */
  int32_t *q_tile_order;  /* [R * ceil(T / VA_TILE)] query tiles in launch order: tiles of the longest examples  */
  int32_t *kv_tile_order; /* first, tiles of one example adjacent, heaviest first; tiles of examples of at most   */
                          /* VA_TILE tokens last, in stream order.  Key tiles likewise.  Entry: tile index in    */
                          /* bits 0..23 (VA_ORDER_TILE), bits 24..30 the tile's head rotation (which head runs   */
                          /* on which XCD: one value per long example, rank / 8 for short ones)                  */
  int32_t *scratch;       /* internal: per-chunk partial scans and tile costs                            */
} va_segments;

/* Bytes of device memory a plan buffer for a [rows, tokens_per_row] stream needs (0 on bad shape). */
size_t va_plan_bytes(int32_t rows, int32_t tokens_per_row);

/* Carve `plan` (device, >= va_plan_bytes, 256-byte aligned) into the arrays of `seg` (host struct).
 * Host-only pointer arithmetic; launches nothing. */
va_status va_segments_bind(void *plan, size_t plan_bytes, int32_t rows, int32_t tokens_per_row,
                           va_segments *seg /* host, out */);

/*
 * position_ids -> cu_seqlens (paper, Section 3: "compute cu_seq_len from position_ids").
 *   position_ids : device, [rows, tokens_per_row] of `it`.  Token t starts an example iff it is
 *                  the first token of its row or its id equals 0; other values are not inspected.
 *   seg          : host struct bound to a plan buffer; all its arrays are written, including
 *                  the tile schedule (which query/key tiles exist and in which order to run them).
 * Integer work only; results are exact.
 */
va_status va_pack_to_cu_seqlens(const void *position_ids, va_itype it, int32_t rows,
                                int32_t tokens_per_row, const va_segments *seg, void *stream);

/*
 * Padding-free collator on the device (paper, Section 3.4; worked example in Section 3.5): the
 * step that produces the position ids the call above consumes.  A minibatch of n_examples
 * examples, held as a padded batch with per-example lengths, is concatenated into ONE packed row
 * of n_out tokens:
 *     input_ids     the tokens of the examples in order
 *     labels        their labels (labels_padded, or the ids when that is NULL) with the first
 *                   label of every example replaced by -100
 *     position_ids  0 .. L-1 inside every example
 *   ids_padded, labels_padded : device, [n_examples, padded_len] of `it`; entries past an example's
 *                   length are never read.  labels_padded may be NULL.
 *   lengths       : device, [n_examples] int32; values outside [0, padded_len] are clamped.
 *   n_out         : tokens in the packed row; normally the sum of the lengths.  If the lengths
 *                   sum to less, the tail is one pad pseudo-example (pad_id, label -100, ids
 *                   0, 1, 2, ...); if to more, the row is cut at n_out (the last example is
 *                   broken, as fixed-length packing does: Table 1).
 *   input_ids, labels, position_ids : device, [n_out] of `it`, fully overwritten.
 *   example_offsets : device, [n_examples + 1] int32: running sum of the clamped lengths
 *                   (example_offsets[n_examples] = their total, not clipped to n_out).
 * n_examples * padded_len must stay below 2^31 - 1 (VA_ERR_SHAPE).  Integer work only; exact.
 */
va_status va_collate_padding_free(const void *ids_padded, const void *labels_padded, va_itype it,
                                  const int32_t *lengths, int32_t n_examples, int32_t padded_len,
                                  int32_t n_out, int64_t pad_id, void *input_ids, void *labels,
                                  void *position_ids, int32_t *example_offsets, void *stream);

/*
 * Rotary position embedding from the same position ids (paper, Section 3: a model that accepts
 * position ids applies them to its positional encoding, so every packed example is encoded as if
 * it were alone).  For each token t, head h and pair c in [0, d/2):
 *     a = position_ids[t] * theta_base^(-2c/d)
 *     y[t,h,c]       = x[t,h,c] cos a - x[t,h,c+d/2] sin a
 *     y[t,h,c + d/2] = x[t,h,c+d/2] cos a + x[t,h,c] sin a
 * ("rotate-half" pairing; the paper fixes neither pairing nor base).
 *   x, y          : device, [n_tokens, heads, d] of `dt`; y may be x (in place).  d even, <= 256.
 *   position_ids  : device, [n_tokens] of `it` (the flattened [rows, tokens_per_row] ids).
 *   theta_base    : <= 0 means 10000.
 *   inverse       : non-zero rotates by -a (the transpose): d(loss)/dx from d(loss)/dy.
 * Angles are formed and range-reduced in fp64, products in fp32; bf16 / fp16 results are rounded to
 * nearest even.  All three element types are accepted.
 */
va_status va_rope_apply(const void *x, void *y, va_dtype dt, const void *position_ids, va_itype it,
                        int32_t n_tokens, int32_t heads, int32_t d, float theta_base, int inverse,
                        void *stream);

/* Workspace bytes for one forward (is_bwd = 0) or backward (is_bwd = 1) call (0 on bad shape). */
size_t va_attn_workspace_bytes(int32_t n_tokens, int32_t hq, int32_t hkv, int32_t d, int is_bwd);

/*
 * Forward: for every example [a, b), head h, token i in [a, b):
 *     S_ij = softmax_scale * q_i . k_j  (a <= j <= i),  P_i = softmax_j(S_i),
 *     O_i = sum_j P_ij v_j,  LSE[h, i] = log sum_j exp(S_ij)   (natural log)
 * (the varlen attention routine the paper's Section 3 hands cu_seqlens to; the mask is
 * Table 1's "correct cross-attention").  Only key tiles that intersect an example's
 * causal triangle are visited.
 *   dt            : element type of Q, K, V, O.  VA_BF16 and VA_F16 with d a multiple of 8 up to 256
 *                   run the MFMA kernels (unrolled for d = 64, 96, 128, 256; a smaller d is padded
 *                   with zero columns on the fly); other (dt, d <= 256) combinations run a plain
 *                   fp32-arithmetic kernel.
 *   softmax_scale : <= 0 means 1 / sqrt(d).
 *   workspace     : >= va_attn_workspace_bytes(..., 0) bytes (may be NULL when that is 0).
 */
va_status va_varlen_attn_fwd(const void *Q, const void *K, const void *V, void *O, float *LSE,
                             const va_segments *seg, int32_t rows, int32_t tokens_per_row,
                             int32_t hq, int32_t hkv, int32_t d, va_dtype dt, float softmax_scale,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward of the above for loss = sum(O * dO), from the saved O and LSE:
 *     P_ij = exp(S_ij - LSE_i),  dP_ij = dO_i . v_j,  D_i = dO_i . O_i,  dS_ij = P_ij (dP_ij - D_i)
 *     dQ_i = scale * sum_j dS_ij k_j
 *     dK_j = scale * sum_{i >= j} dS_ij q_i,   dV_j = sum_{i >= j} P_ij dO_i
 * with dK, dV also summed over the Hq / Hkv query heads of a KV head.  Same mask, same
 * skipped tiles.  Results are deterministic (no atomics).  The 16-bit kernels accumulate in fp32;
 * they take D from the row sums of dS (which removes the rounding of the stored O) and carry the
 * large entries of P and dS through the matrix units in two 16-bit parts.
 *   grad_dt   : element type of dQ, dK, dV: VA_F32, or the 16-bit type of the inputs (VA_BF16 also
 *               with fp32 inputs); other pairs: VA_ERR_UNSUPPORTED.
 *   workspace : >= va_attn_workspace_bytes(..., 1) bytes (holds D, [Hq, N] float).
 */
va_status va_varlen_attn_bwd(const void *dO, const void *Q, const void *K, const void *V,
                             const void *O, const float *LSE, void *dQ, void *dK, void *dV,
                             va_dtype grad_dt, const va_segments *seg, int32_t rows,
                             int32_t tokens_per_row, int32_t hq, int32_t hkv, int32_t d,
                             va_dtype dt, float softmax_scale, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * The backward above for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as va_varlen_attn_bwd, without `workspace`: D lives in a device array inside the library
 * (VA_NOALLOC_SCRATCH_BYTES per GPU, held until the process ends).  Calls no hipMalloc / hipFree and no
 * allocating routine; the first call on a device looks the array's address up once (make that call
 * outside stream capture).
 *   Limit: rows * tokens_per_row * hq * 4 <= VA_NOALLOC_SCRATCH_BYTES, else VA_ERR_WORKSPACE and
 *   nothing is enqueued.
 *   All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *   streams, or threads) race; calls enqueued on one stream are safe.
 */
#define VA_NOALLOC_SCRATCH_BYTES (32u << 20)
va_status va_varlen_attn_bwd_noalloc(const void *dO, const void *Q, const void *K, const void *V,
                                     const void *O, const float *LSE, void *dQ, void *dK, void *dV,
                                     va_dtype grad_dt, const va_segments *seg, int32_t rows,
                                     int32_t tokens_per_row, int32_t hq, int32_t hkv, int32_t d,
                                     va_dtype dt, float softmax_scale, void *stream);

/*
 * The backward in parts, so that a caller can time its kernels one by one with events on `stream`:
 * `stages` is an OR of the flags below.
 *   VA_STAGE_D    D = rowsum(dO * O) into `workspace`.
 *   VA_STAGE_DQ   dQ.  The plain kernels read D from `workspace`; the MFMA kernel forms D for its
 *                 own rows and (re)writes `workspace` with it - refined by the row sums of dS, which
 *                 take out the rounding of the stored O (so dK/dV are most accurate after this stage).
 *   VA_STAGE_DKDV dK, dV; reads the D that an earlier VA_STAGE_D or VA_STAGE_DQ left in `workspace`.
 * Within one call the order is D (skipped when the MFMA dQ kernel makes it redundant), dQ, dK/dV;
 * all three flags give exactly va_varlen_attn_bwd.
 * The MFMA dK/dV kernel has two workgroup shapes (head_dim <= 128): 128-key tiles for batches of long
 * examples, 64-key tiles otherwise.  By default both are enqueued and the device picks by the batch's
 * mean example length (the host never sees the lengths); the other's workgroups leave at once.  A
 * caller that knows its lengths can add ONE of
 *   VA_HINT_LONG_EXAMPLES   mean example length >= 1024 tokens: only the 128-key shape is enqueued
 *   VA_HINT_SHORT_EXAMPLES  otherwise: only the 64-key shape
 * Either shape computes every result whatever the lengths; a wrong hint costs speed only.
 * Arguments, validation and errors as va_varlen_attn_bwd; no stage bit, both hints or unknown bits:
 * VA_ERR_UNSUPPORTED.
 */
#define VA_STAGE_D 1u
#define VA_STAGE_DKDV 2u
#define VA_STAGE_DQ 4u
#define VA_HINT_LONG_EXAMPLES 8u
#define VA_HINT_SHORT_EXAMPLES 16u
va_status va_varlen_attn_bwd_stages(const void *dO, const void *Q, const void *K, const void *V,
                                    const void *O, const float *LSE, void *dQ, void *dK, void *dV,
                                    va_dtype grad_dt, const va_segments *seg, int32_t rows,
                                    int32_t tokens_per_row, int32_t hq, int32_t hkv, int32_t d,
                                    va_dtype dt, float softmax_scale, void *workspace,
                                    size_t workspace_bytes, void *stream, uint32_t stages);

/* Static string for a status code. */
const char *va_status_string(va_status s);

/* Library version string (host). */
const char *va_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VARLEN_ATTN_H */
