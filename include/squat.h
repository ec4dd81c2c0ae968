/*
 * squat.h -- C ABI of the MI355X (gfx950) implementation of the SQuat
 * key-quantization path (arxiv 2503.24358, "SQuat: Subspace-orthogonal KV
 * Cache Quantization").
 *
 * Four calls cover the path, in the order Algorithm 1 uses them:
 *
 *   squat_build_subspace   prompt queries -> Qhat            (Section 3.2)
 *   squat_prepare          Qhat, lambda, g -> update matrix  (Lemma 2, Lemma 3)
 *   squat_quantize_keys    keys, update matrix -> codes      (Algorithm 1, Quant)
 *   squat_dequantize_keys  codes -> keys                     (Section 2, deq)
 *
 * squat_key_scores is the decode-side consumer of that store (attention
 * logits straight from the codes); squat_key_scores_per_channel is the same
 * for the per-channel store, squat_key_scores_rope for keys stored before the
 * rotary position embedding.
 *
 * squat_quantize_keys groups every key's channels (statistics per token); the
 * pair squat_quantize_keys_per_channel / squat_dequantize_keys_per_channel is
 * the paper's own grouping (statistics per channel over 32 tokens), with the
 * same Qhat and update matrix.
 *
 * Conventions that hold for every call
 *   - Every data pointer is a DEVICE pointer owned by the caller, valid on the
 *     device that is current when the call is made.  Only `ws` buffers are
 *     scratch; everything else is either read-only input or fully overwritten
 *     output.  Inputs and outputs must not alias.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  The calls never synchronise, never allocate or
 *     free device memory and keep no state between calls, so they may be used
 *     from several host threads on different streams.  Buffers must stay alive
 *     until the stream has passed the enqueued work.
 *   - Arguments are validated on the host BEFORE anything is launched.  The
 *     return value is SQUAT_OK (0) or a negative squat_status; on error nothing
 *     was enqueued.  squat_strerror() names a status.
 *   - Row-major tensors; strides are given in ELEMENTS of the tensor's dtype.
 *   - Head size d must be 128 in this version.  "Heads" are independent
 *     problems: several layers may be stacked along the head axis in one call.
 */
#ifndef SQUAT_H
#define SQUAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum squat_dtype {
    SQUAT_F32 = 0,   /* IEEE binary32 */
    SQUAT_F16 = 1,   /* IEEE binary16 */
    SQUAT_BF16 = 2   /* bfloat16 */
} squat_dtype;

typedef enum squat_status {
    SQUAT_OK = 0,
    SQUAT_E_NULLPTR = -1,   /* a required pointer is NULL */
    SQUAT_E_BADSHAPE = -2,  /* unsupported d, r, g, G, bits, negative sizes, bad strides */
    SQUAT_E_BADDTYPE = -3,  /* dtype not one of squat_dtype / not allowed for this tensor */
    SQUAT_E_ALIGN = -4,     /* pointer or stride breaks the stated alignment */
    SQUAT_E_WORKSPACE = -5, /* ws is NULL or ws_bytes too small */
    SQUAT_E_HIP = -6,       /* the HIP runtime refused a launch (hipGetLastError) */
    SQUAT_E_BADVALUE = -7   /* lambda negative or NaN */
} squat_status;

typedef void* squat_stream; /* hipStream_t */

/* Library version: major * 10000 + minor * 100 + patch. */
int squat_version(void);

/* Static, human-readable name of a status code (never NULL). */
const char* squat_strerror(int status);

/* ------------------------------------------------------------------------- *
 * squat_build_subspace  (Section 3.2, last paragraph; Algorithm 1, the SVD
 * line and the line defining Qhat; GQA pooling: appendix "Details of Our Main
 * Algorithm").
 *
 * For every KV head j, pools the prompt queries of its q_per_kv query heads
 * (query heads j*q_per_kv .. (j+1)*q_per_kv-1) row-wise, forms their Gram
 * matrix Q^T Q, takes its r largest eigenpairs (eig_i, v_i) and writes
 *     qhat[j, i, :] = sqrt(eig_i) * v_i,       i = 0..r-1, descending eig,
 * i.e. the top-r right singular vectors of the pooled queries scaled by their
 * singular values.  Each row's sign is fixed so that its largest-magnitude
 * component is positive.  Eigenvalues that are zero (r > rank) give zero rows.
 *
 *   q       [n_kv_heads*q_per_kv, n_tokens, d] dtype q_dt, element (h,t,c) at
 *           q[h*q_stride_head + t*q_stride_token + c]; base pointer 16-byte
 *           aligned, both strides multiples of 8 elements; a token stride of
 *           2^27 bytes or more is SQUAT_E_BADSHAPE.
 *   qhat    out [n_kv_heads, r, d] float, dense.  May be NULL only if r == 0.
 *   eig     out [n_kv_heads, r] float, eigenvalues of Q^T Q (squared singular
 *           values), descending.  May be NULL.
 *   gram    out [n_kv_heads, d, d] float, the pooled Gram matrix.  May be NULL.
 *   ws      scratch of at least squat_build_subspace_workspace(...) bytes,
 *           256-byte aligned.
 *   0 <= r <= d.  n_tokens >= 1.  The Gram products are exact for bf16/f16
 *   inputs and accumulate in fp32 within a slab of tokens, fp64 across slabs;
 *   the eigen-solver works in fp64 (r <= 64: Householder tridiagonalisation,
 *   Sturm-count search, inverse iteration, the vectors in batches of 32;
 *   otherwise, or if that route's own checks fail for a head, cyclic
 *   one-sided Jacobi).
 * ------------------------------------------------------------------------- */
size_t squat_build_subspace_workspace(int64_t n_tokens, int n_kv_heads, int q_per_kv, int d, int r);

int squat_build_subspace(const void* q, squat_dtype q_dt, int64_t n_tokens, int n_kv_heads,
                         int q_per_kv, int d, int64_t q_stride_head, int64_t q_stride_token,
                         int r, float* qhat, float* eig, float* gram,
                         void* ws, size_t ws_bytes, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_refresh_subspace  (Algorithm 1, prefill phase, the remark on the SVD
 * line: the decomposition "can be accelerated using block power method";
 * Section 3.2 for what Qhat is; GQA pooling as for squat_build_subspace).
 *
 * The cheaper, approximate route to Qhat, and the way to keep Qhat current
 * while queries keep arriving.  The caller owns a running Gram matrix per KV
 * head (`gram_state`, fp64); the call
 *   1. adds the pooled Gram matrix of `q_new` to it (accumulate != 0) or
 *      overwrites it with that matrix (accumulate == 0); n_new == 0 with
 *      accumulate != 0 leaves it as it is;
 *   2. iterations >= 0: runs that many steps X <- orth(G X) of block power
 *      iteration on a block of 32 vectors, started from the non-zero rows of
 *      `qhat_prev` (normalised) completed with coordinate vectors e_c,
 *      c = 0, s, 2 s, ... (s = d / number of missing columns), and takes the
 *      Ritz pairs (theta_i, x_i) of the final block (Rayleigh-Ritz):
 *          qhat[j, i, :] = sqrt(theta_i) x_i,  i = 0..r-1, descending theta,
 *      sign convention as squat_build_subspace.  The iteration converges like
 *      (eig_33 / eig_r)^iterations: fast for queries that concentrate in a
 *      low-dimensional subspace and for warm starts, not at all for a flat
 *      spectrum; `residual` reports how far it got.  A head whose block turns
 *      out rank-deficient is redone by the exact solver (residual 0).
 *      iterations < 0: the exact solver of squat_build_subspace on the state.
 *
 *   q_new    [n_kv_heads*q_per_kv, n_new, d] as `q` of squat_build_subspace
 *            (same alignment rules); may be NULL if n_new == 0.
 *   gram_state  in/out [n_kv_heads, d, d] double, dense, 16-byte aligned.
 *   r        0 <= r <= 32 for iterations >= 0 (r <= d otherwise).
 *   qhat_prev   [n_kv_heads, r_prev, d] float or NULL (cold start); r_prev <= 32;
 *            may be the same buffer as qhat when r_prev == r.
 *   qhat, eig   as for squat_build_subspace (eig = Ritz values).
 *   residual out [n_kv_heads] float or NULL: max over the r pairs of
 *            ||G x_i - theta_i x_i||_2 / theta_1.
 *   ws       scratch of at least squat_refresh_subspace_workspace(...) bytes,
 *            256-byte aligned.
 * ------------------------------------------------------------------------- */
size_t squat_refresh_subspace_workspace(int64_t n_new, int n_kv_heads, int q_per_kv, int d, int r);

int squat_refresh_subspace(const void* q_new, squat_dtype q_dt, int64_t n_new, int n_kv_heads, int q_per_kv,
                           int d, int64_t q_stride_head, int64_t q_stride_token, int accumulate,
                           double* gram_state, int r, int iterations, const float* qhat_prev, int r_prev,
                           float* qhat, float* eig, float* residual, void* ws, size_t ws_bytes,
                           squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_prepare  (Lemma 2: the block update B_t H_t; Lemma 3 and its Remark:
 * the A_t^{-1} chain; Prop. 1 is the g = 1 case).
 *
 * For every head writes the d x d matrix U, row-major, with
 *     U[t*g : d, (t-1)*g : t*g] = B_t H_t          for t = 1 .. d/g - 1
 * and zeros everywhere else, where P_inv = (I + lambda Qhat^T Qhat)^{-1},
 * A_t is its leading (t g x t g) block, B_t the block below it and H_t the
 * last g columns of A_t^{-1}.  The kernel evaluates the equivalent rank-r
 * form  -Qr^T (I/lambda + Qr Qr^T)^{-1} Qb  (Qb, Qr: the columns of Qhat in
 * and after block t) in fp64 (r <= 64 and finite lambda: by a Cholesky
 * factorisation, heads that turn out ill-conditioned and all other cases by an
 * eigen-decomposition).  lambda = +INFINITY selects the limit
 * -pinv(Qr) Qb (the equality constraint of Eq. (1)); lambda = 0 or r = 0
 * gives U = 0 (plain round-to-nearest).  Every entry is rounded to the nearest
 * fp16-representable number (relative 2^-12, entries must stay below 65504)
 * and stored as fp32: squat_quantize_keys detects such a matrix and contracts
 * with two fp16 matrix passes instead of three.
 *
 *   qhat    [n_heads, r, d] float, dense (NULL allowed only if r == 0).
 *   update  out [n_heads, d, d] float, dense, 16-byte aligned.
 *   g       32, 64 or 128 (g = 128 = d means a single block: U = 0).
 *   ws      scratch of at least squat_prepare_workspace(...) bytes, 256-byte
 *           aligned.
 * ------------------------------------------------------------------------- */
size_t squat_prepare_workspace(int n_heads, int d, int r, int g);

int squat_prepare(const float* qhat, int n_heads, int d, int r, float lambda, int g,
                  float* update, void* ws, size_t ws_bytes, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_prepare_ex  (Lemma 2, Lemma 3: as squat_prepare) -- squat_prepare with
 * a choice of how the entries of U are stored.
 *
 *   flags   0: as squat_prepare, entries on the fp16 grid (an approximation of
 *           this implementation, relative 2^-12 per entry, in exchange for a
 *           two-pass contraction in the quantize kernels);
 *           SQUAT_PREPARE_FULL_PRECISION: the fp64 result rounded once to fp32
 *           (Lemma 2's matrix to fp32 accuracy; the quantize kernels then run
 *           their three-pass contraction, a few per cent slower).
 *           Any other bit set: SQUAT_E_BADVALUE.
 *   Everything else as for squat_prepare (same workspace size).
 * ------------------------------------------------------------------------- */
#define SQUAT_PREPARE_FULL_PRECISION 1u

int squat_prepare_ex(const float* qhat, int n_heads, int d, int r, float lambda, int g, unsigned flags,
                     float* update, void* ws, size_t ws_bytes, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_prepare_noalloc  -- squat_prepare for callers that cannot allocate or
 * carry a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.
 *
 * Same arguments, checks, kernels and results as squat_prepare, without `ws`:
 * the scratch is a 4 MiB array inside the library's code object (one copy per
 * device, held until the process ends).  The call allocates and frees nothing.
 * Limits: r <= 32 with a finite lambda needs 4 bytes per head (n_heads <=
 * 2^20); r <= 32 with lambda = +INFINITY needs none; r > 32 needs
 * n_heads * (d/g - 1) * (r rounded up to even) * (g + d) * 8 bytes, rounded up
 * to 256, plus, for r <= 64 with a finite lambda, 4 bytes per head rounded up
 * to 256.  A problem beyond 4 MiB returns SQUAT_E_WORKSPACE (nothing launched).
 * Every call on a device shares that device's array: calls that may overlap
 * on one device (different streams, or threads) race; order them.  The first
 * call on a device looks the array's address up (no allocation); make that
 * call outside a graph capture.
 * ------------------------------------------------------------------------- */
int squat_prepare_noalloc(const float* qhat, int n_heads, int d, int r, float lambda, int g,
                          float* update, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_quantize_keys  (Section 2 "Quantization": qtz/deq; Algorithm 1,
 * function Quant; Lemma 2, the update of the not-yet-quantized elements).
 *
 * For every key vector k (one token of one head of one batch entry) runs, on a
 * working copy in fp32: for t = 1 .. d/g, quantize the g channels of block t
 * from their CURRENT values with asymmetric min/max b-bit round-to-nearest
 * (per token, over groups of `group` consecutive channels; scale and zero are
 * rounded to fp16 before they are used, ties round to even, codes are clamped
 * to [0, 2^b-1], a constant group has scale 0 and codes 0), freeze them at
 * their dequantized values, and if t < d/g add  U[t g:, block] * (deq - current)
 * to the remaining channels.  update == NULL is plain round-to-nearest.
 * When group > g the statistics of a group are taken once, when its first
 * block is reached.
 *
 *   k        [n_batch, n_heads, n_tokens, d] dtype k_dt; element (b,h,t,c) at
 *            k[b*k_stride_batch + h*k_stride_head + t*k_stride_token + c];
 *            base 16-byte aligned, strides multiples of 8 elements (a token
 *            stride of 2^26 bytes or more is SQUAT_E_BADSHAPE).  Not modified.
 *   update   [n_heads, d, d] float as written by squat_prepare (same g), or
 *            any fp32 matrix of that block structure with |entries| < 65504, or
 *            NULL.  update_stride_batch (elements) is added per batch entry;
 *            0 shares one matrix per head across the batch (the paper's
 *            batch > 1 rule).
 *   bits     2 or 4.   group  32, 64 or 128.   g  32, 64 or 128; group must
 *            divide g or g must divide group.
 *   codes    out [n_batch, n_heads, n_tokens, d*bits/32] uint32, dense,
 *            16-byte aligned.  Channel c of a key is in word c / (32/bits) at
 *            bit offset bits * (c mod 32/bits).
 *   scale    out [n_batch, n_heads, n_tokens, d/group] fp16 bit patterns.
 *   zero     out, same shape: the (real-valued) zero-point m.
 *   n_tokens may be any value >= 0 (0: nothing is launched).
 * ------------------------------------------------------------------------- */
int squat_quantize_keys(const void* k, squat_dtype k_dt, int64_t n_batch, int n_heads,
                        int64_t n_tokens, int d, int64_t k_stride_batch, int64_t k_stride_head,
                        int64_t k_stride_token, const float* update, int64_t update_stride_batch,
                        int bits, int group, int g, uint32_t* codes, uint16_t* scale,
                        uint16_t* zero, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_quantize_keys_plan  (Algorithm 1, prefill phase: the token groups of a
 * prompt are quantized in parallel -- this says how a call spreads them).
 *
 * Host-only query, nothing is launched: the launch shape squat_quantize_keys
 * (per_channel = 0) or squat_quantize_keys_per_channel (per_channel = 1) uses
 * for a problem of this size on the current device.  Keys are processed in
 * tiles of 32 consecutive tokens of one (batch entry, head).  The tiles that
 * share an update matrix (a head's, over the whole batch, or one batch
 * entry's when update_stride_batch != 0) form a "problem"; each problem gets
 * workgroups_per_problem persistent workgroups (as many as fill the device
 * once, at most one per tile) whose wavefronts take tiles
 *     w, w + S, w + 2 S, ...     (w = wavefront_in_workgroup *
 *     workgroups_per_problem + workgroup_in_problem,
 *     S = workgroups_per_problem * wavefronts_per_workgroup)
 * until tiles_per_problem is reached.  A wavefront therefore runs
 * floor(tiles_per_problem / S) or one more tile, and a problem with fewer
 * tiles than S leaves the higher-numbered wavefronts of every workgroup idle
 * rather than whole workgroups.
 *
 *   has_update   0 for update == NULL.   out   host memory.
 *   Same argument checks (and status codes) as the quantize call itself.
 * ------------------------------------------------------------------------- */
typedef struct squat_quantize_plan {
    int64_t problems;
    int workgroups_per_problem;
    int wavefronts_per_workgroup;
    int64_t tiles_per_problem;
} squat_quantize_plan;

int squat_quantize_keys_plan(squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens,
                             int has_update, int64_t update_stride_batch, int bits, int group, int g,
                             int per_channel, squat_quantize_plan* out);

/* ------------------------------------------------------------------------- *
 * squat_dequantize_keys  (Section 2: deq(c) = c * Delta + m).
 *
 * Inverse of the storage format above: k_out[b,h,t,c] = code * scale + zero
 * of the group of channel c, computed in fp32 (one fused multiply-add) and
 * rounded once to out_dt.
 *
 *   codes, scale, zero   as written by squat_quantize_keys (dense).
 *   k_out   [n_batch, n_heads, n_tokens, d] dtype out_dt with strides in
 *           elements (multiples of 8, base 16-byte aligned).
 * ------------------------------------------------------------------------- */
int squat_dequantize_keys(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                          int64_t n_batch, int n_heads, int64_t n_tokens, int d, int bits,
                          int group, void* k_out, squat_dtype out_dt, int64_t o_stride_batch,
                          int64_t o_stride_head, int64_t o_stride_token, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_quantize_keys_per_channel  (Algorithm 1, function Quant, as printed:
 * "per-channel" quantization of each key block; Section 2 "Quantization";
 * Section 4 "Hyper-parameters": group size 32 = residual length 32; Lemma 2
 * for the update).
 *
 * Tokens are taken in groups of `group` = 32 consecutive tokens of one head
 * (what the decode phase flushes from the residual buffer, or 32-token slices
 * of the prompt).  For one such group, on a working copy in fp32: for
 * t = 1 .. d/g, every channel of block t is quantized on its own over the 32
 * tokens, from their CURRENT values, with asymmetric min/max b-bit
 * round-to-nearest (scale and zero rounded to fp16 before use, ties to even,
 * codes clamped to [0, 2^b-1], a constant channel has scale 0 and codes 0);
 * the block is frozen at its dequantized values and, if t < d/g, every token's
 * remaining channels receive  U[t g:, block] * (deq - current)  of that token.
 * update == NULL is plain per-channel round-to-nearest (KIVI's key format).
 *
 *   k, update, update_stride_batch, bits, g    as for squat_quantize_keys.
 *   group    must be 32.   n_tokens must be a multiple of 32 (the caller keeps
 *            the remainder in its 16-bit residual buffer, as Algorithm 1 does).
 *   codes    out [n_batch, n_heads, n_tokens/32, d, bits] uint32, dense,
 *            16-byte aligned: the 32 codes of channel c in token group T are
 *            `bits` consecutive words; token j of the group is in word
 *            j / (32/bits) at bit offset bits * (j mod 32/bits).
 *   scale    out [n_batch, n_heads, n_tokens/32, d] fp16 bit patterns,
 *            4-byte aligned.
 *   zero     out, same shape: the (real-valued) zero-point m.
 *   Keys must be finite: a NaN or Inf spoils the whole group of 32 tokens.
 * ------------------------------------------------------------------------- */
int squat_quantize_keys_per_channel(const void* k, squat_dtype k_dt, int64_t n_batch, int n_heads,
                                    int64_t n_tokens, int d, int64_t k_stride_batch,
                                    int64_t k_stride_head, int64_t k_stride_token,
                                    const float* update, int64_t update_stride_batch, int bits,
                                    int group, int g, uint32_t* codes, uint16_t* scale,
                                    uint16_t* zero, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_dequantize_keys_per_channel  (Section 2: deq(c) = c * Delta + m, on
 * the per-channel store).
 *
 * k_out[b,h,t,c] = code * scale + zero of (token group t / 32, channel c), one
 * fused multiply-add in fp32, rounded once to out_dt.
 *
 *   codes, scale, zero   as written by squat_quantize_keys_per_channel (dense;
 *           all three 16-byte aligned).
 *   group   must be 32; n_tokens a multiple of 32.
 *   k_out   [n_batch, n_heads, n_tokens, d] dtype out_dt with strides in
 *           elements (multiples of 8, base 16-byte aligned).
 * ------------------------------------------------------------------------- */
int squat_dequantize_keys_per_channel(const uint32_t* codes, const uint16_t* scale,
                                      const uint16_t* zero, int64_t n_batch, int n_heads,
                                      int64_t n_tokens, int d, int bits, int group, void* k_out,
                                      squat_dtype out_dt, int64_t o_stride_batch,
                                      int64_t o_stride_head, int64_t o_stride_token,
                                      squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_key_scores  (decoding phase of Algorithm 1: attention over the keys
 * that have left the residual buffer, which exist only in quantized form;
 * Section 2: deq(c) = c * Delta + m).
 *
 * scores[b, hq, t] = out_scale * sum_c q[b, hq, c] * (code[b, h, t, c] * scale + zero)
 * for the KV head h = hq / q_per_kv, read straight from the packed store of
 * squat_quantize_keys (per-token groups) without materialising the keys.  The
 * caller computes the logits of its full-precision residual tokens itself and
 * places them behind these (hence the output strides).
 *
 *   codes, scale, zero   as written by squat_quantize_keys: [n_batch,
 *            n_kv_heads, n_tokens, ...], dense; codes 16-byte, scale/zero
 *            8-byte aligned.  n_tokens < 2^25.  (Fastest when every (batch,
 *            head) row block of scale and zero starts on a 16-byte boundary,
 *            i.e. both bases 16-byte aligned and n_tokens * 2 * d / group a
 *            multiple of 16: whole 16-token units are then fetched with
 *            16-byte loads; otherwise every lane fetches its own pieces.  The
 *            results are the same.)
 *   q        [n_batch, n_kv_heads*q_per_kv, d] dtype q_dt, element (b,hq,c) at
 *            q[b*q_stride_batch + hq*q_stride_head + c]; base 16-byte aligned,
 *            strides multiples of 8 elements; |q| < 16000.
 *   q_per_kv 1 .. 8 query heads per KV head.
 *   out_scale  e.g. 1/sqrt(d); must not be NaN.
 *   scores   out, float: element (b,hq,t) at scores[b*s_stride_batch +
 *            hq*s_stride_head + t]; s_stride_head >= n_tokens.
 *   Products of queries and codes are exact (fp16 high/low query parts times
 *   integer codes on the matrix cores), sums are fp32.
 * ------------------------------------------------------------------------- */
int squat_key_scores(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                     int64_t n_batch, int n_kv_heads, int64_t n_tokens, int d, int bits, int group,
                     const void* q, squat_dtype q_dt, int q_per_kv, int64_t q_stride_batch,
                     int64_t q_stride_head, float out_scale, float* scores,
                     int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_key_scores_rope  (Section 4: the pre-RoPE variant, which quantizes and
 * stores keys before the rotary position embedding and applies positions on
 * the fly after dequantization; Section 2: deq).
 *
 * scores[b, hq, t] = out_scale * sum_c q[b, hq, c] * RoPE_{pos0 + t}(deq(code[b, h, t, :]))[c]
 * for the KV head h = hq / q_per_kv, where RoPE_p rotates every channel pair
 * (c, c + 64), c < 64, by the angle p * inv_freq[c]:
 *     x'_c = x_c cos - x_{c+64} sin,    x'_{c+64} = x_{c+64} cos + x_c sin.
 * The queries are taken as given (already rotated to their own position).
 *
 *   codes, scale, zero, q, q_per_kv, out_scale, scores and the strides   as for
 *            squat_key_scores (per-token store).
 *   inv_freq [64] float, device memory: the rotary frequencies (theta^(-c/64),
 *            or any scaled variant).
 *   pos0     position of token 0 of the store, 0 <= pos0 < 2^40.
 *   Accuracy: the queries enter as exact fp16 high/low pairs (rotated in fp32
 *   by the part of the angle that a block of 64 tokens shares, angles good to
 *   ~1e-5 rad); the key is dequantized and rotated in packed fp16, where the
 *   dequantized value, the cos/sin entry, one product and the result are each
 *   rounded to fp16: a rotated channel is off by at most 4 * 2^-11 times the
 *   norm of its rotary pair (typically a quarter of that), a logit by at most
 *   4 * 2^-11 * out_scale * sum_{c<64} (|q_c| + |q_{c+64}|) |(k_c, k_{c+64})|.
 *   Dequantized keys and their rotations must stay below 65504.
 * ------------------------------------------------------------------------- */
int squat_key_scores_rope(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                          int64_t n_batch, int n_kv_heads, int64_t n_tokens, int d, int bits, int group,
                          const float* inv_freq, int64_t pos0, const void* q, squat_dtype q_dt,
                          int q_per_kv, int64_t q_stride_batch, int64_t q_stride_head, float out_scale,
                          float* scores, int64_t s_stride_batch, int64_t s_stride_head,
                          squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_key_scores_per_channel  (decoding phase of Algorithm 1 with the
 * grouping its Quant function prints; Section 2: deq(c) = c * Delta + m).
 *
 * scores[b, hq, t] = out_scale * sum_c q[b, hq, c] * (code * scale + zero) with
 * the scale and zero-point of (token group t / 32, channel c), read straight
 * from the packed store of squat_quantize_keys_per_channel.
 *
 *   codes, scale, zero   as written by squat_quantize_keys_per_channel, dense,
 *            all three 16-byte aligned.  group must be 32, n_tokens a multiple
 *            of 32 and < 2^25.
 *   q, q_per_kv, out_scale, scores and their strides   as for squat_key_scores;
 *            |q| is not restricted (the kernel normalises by the exponent of
 *            the largest |q| of a KV head, and per token group by the exponent
 *            of its largest scale).
 *   Each product q_c * scale_c is carried as an fp16 high/low pair: relative
 *   error below 2^-21 per term, and an absolute floor of 2^-24 times (largest
 *   |q| of the KV head) x (largest scale of the token group) per term; products
 *   with the integer codes are exact, sums are fp32.
 * ------------------------------------------------------------------------- */
int squat_key_scores_per_channel(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                                 int64_t n_batch, int n_kv_heads, int64_t n_tokens, int d, int bits,
                                 int group, const void* q, squat_dtype q_dt, int q_per_kv,
                                 int64_t q_stride_batch, int64_t q_stride_head, float out_scale,
                                 float* scores, int64_t s_stride_batch, int64_t s_stride_head,
                                 squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_key_scores_rope_per_channel  (Section 4: the pre-RoPE variant, rotation
 * after dequantization, on the grouping Algorithm 1's Quant function prints:
 * the combination the paper's main tables report as SQuat-pre).
 *
 * scores[b, hq, t] = out_scale * sum_c q[b, hq, c] * RoPE_{pos0 + t}(deq(t, :))[c]
 * with deq(t, c) = code * scale + zero of (token group t / 32, channel c) and
 * RoPE as for squat_key_scores_rope.
 *
 *   codes, scale, zero   as written by squat_quantize_keys_per_channel, dense,
 *            all three 16-byte aligned.  group must be 32, n_tokens a multiple
 *            of 32 and < 2^25.
 *   inv_freq, pos0   as for squat_key_scores_rope.
 *   q, q_per_kv, out_scale, scores and their strides   as for squat_key_scores
 *            (|q| below the fp16 range, 65504).
 *   Accuracy: as squat_key_scores_rope.
 * ------------------------------------------------------------------------- */
int squat_key_scores_rope_per_channel(const uint32_t* codes, const uint16_t* scale, const uint16_t* zero,
                                      int64_t n_batch, int n_kv_heads, int64_t n_tokens, int d, int bits,
                                      int group, const float* inv_freq, int64_t pos0, const void* q,
                                      squat_dtype q_dt, int q_per_kv, int64_t q_stride_batch,
                                      int64_t q_stride_head, float out_scale, float* scores,
                                      int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream);

/* ------------------------------------------------------------------------- *
 * squat_cache_*  (Algorithm 1: the prefill split "r = l mod R", the residual
 * buffer K^full and its flush in the decoding phase; appendix "Details of Our
 * Main Algorithm": values follow KIVI, per-token groups, the most recent R
 * tokens in full precision, the oldest one quantized when token R + 1 arrives).
 *
 * A small STATEFUL object on top of the stateless calls: it owns no device
 * memory (everything lives in one caller-provided arena) and holds only
 * counters and pointers on the host.  All sequences of the batch advance
 * together.  Calls enqueue on the given stream and update the counters when
 * they are made: use one stream and one host thread per cache.
 *
 *   keys    quantized with squat_quantize_keys (per-token groups, the update
 *           matrix given at creation, shared by the batch) in groups of
 *           `residual` tokens; the rest waits in the residual buffer.
 *   values  (optional) quantized with plain round-to-nearest one token at a
 *           time once they are older than `residual` tokens.
 *   keys    with key_per_channel: quantized with squat_quantize_keys_per_channel
 *           instead (groups of 32 tokens per channel, the paper's grouping).
 *   logits  squat_cache_key_scores (squat_cache_key_scores_rope for keys stored before the rotary embedding)
 *           = squat_key_scores (or _per_channel; or _rope) over the quantized keys
 *           followed by plain dot products over the residual keys:
 *           scores[b, hq, 0 .. keys_quantized + keys_residual).
 * ------------------------------------------------------------------------- */
typedef struct squat_cache squat_cache;

typedef struct squat_cache_config {
    int64_t n_batch;
    int n_kv_heads;       /* layers may be stacked along this axis */
    int q_per_kv;         /* 1 .. 8 */
    int d;                /* 128 */
    int bits;             /* 2 or 4 */
    int group;            /* channels per quantization group: 32, 64 or 128 */
    int g;                /* channels frozen per iteration: 32, 64 or 128 (as given to squat_prepare) */
    int residual;         /* R: full-precision tokens kept; 1 .. 1024 (32 in the paper) */
    int64_t max_tokens;   /* capacity of the quantized stores per sequence; multiple of residual, < 2^25 */
    squat_dtype kv_dtype; /* dtype of incoming keys / values and of the residual buffers */
    int quantize_values;  /* 0: keys only */
    int key_per_channel;  /* 0: keys grouped per token (squat_quantize_keys, `group` channels per group);
                             1: keys grouped per channel over 32 tokens as Algorithm 1 prints it
                             (squat_quantize_keys_per_channel; residual must be a multiple of 32, the
                             key stores then have the per-channel layout and `group` applies to the
                             values only) */
} squat_cache_config;

typedef struct squat_cache_buffers {   /* device pointers inside the arena */
    uint32_t* key_codes;      /* [n_batch, n_kv_heads, max_tokens, d*bits/32]; per-channel keys:
                                 [n_batch, n_kv_heads, max_tokens/32, d, bits] */
    uint16_t* key_scale;      /* [n_batch, n_kv_heads, max_tokens, d/group]; per-channel keys:
                                 [n_batch, n_kv_heads, max_tokens/32, d] */
    uint16_t* key_zero;
    void* key_residual;       /* [n_batch, n_kv_heads, residual, d] kv_dtype; slots 0 .. keys_residual-1 in use */
    uint32_t* value_codes;    /* same shapes; NULL without values */
    uint16_t* value_scale;
    uint16_t* value_zero;
    void* value_residual;     /* ring: oldest token in slot value_ring_head */
} squat_cache_buffers;

typedef struct squat_cache_counts {
    int64_t n_tokens;         /* tokens seen per sequence */
    int64_t keys_quantized;
    int keys_residual;
    int64_t values_quantized;
    int values_residual;
    int value_ring_head;
} squat_cache_counts;

/* Bytes of device memory the cache needs (0 if the configuration is not supported). */
size_t squat_cache_arena_bytes(const squat_cache_config* cfg);

/* arena: device memory, 256-byte aligned, at least squat_cache_arena_bytes(cfg); update: [n_kv_heads, d, d]
 * float as written by squat_prepare with the same g (NULL: plain round-to-nearest); both must outlive the
 * cache.  *out receives the object (host memory; release it with squat_cache_destroy). */
int squat_cache_create(const squat_cache_config* cfg, void* arena, size_t arena_bytes, const float* update,
                       squat_cache** out);
void squat_cache_destroy(squat_cache* cache);
int squat_cache_reset(squat_cache* cache);          /* forget all tokens (no device work) */
int squat_cache_state(const squat_cache* cache, squat_cache_counts* out);
int squat_cache_get_buffers(const squat_cache* cache, squat_cache_buffers* out);

/* Prompt keys (and values, if configured): [n_batch, n_kv_heads, n_tokens, d] kv_dtype with element strides
 * (multiples of 8, base 16-byte aligned; values use the same strides).  Only on an empty cache.  Keys
 * 0 .. n_tokens - (n_tokens mod residual) - 1 are quantized, the rest goes to the residual buffer. */
int squat_cache_prefill(squat_cache* cache, const void* k, const void* v, int64_t n_tokens,
                        int64_t stride_batch, int64_t stride_head, int64_t stride_token, squat_stream stream);

/* One decoded token per sequence: k, v [n_batch, n_kv_heads, d].  SQUAT_E_BADSHAPE when a store is full. */
int squat_cache_append(squat_cache* cache, const void* k, const void* v, int64_t stride_batch,
                       int64_t stride_head, squat_stream stream);

/* Logits of q [n_batch, n_kv_heads*q_per_kv, d] against every cached key, quantized ones first; arguments
 * as for squat_key_scores; s_stride_head >= keys_quantized + keys_residual. */
int squat_cache_key_scores(const squat_cache* cache, const void* q, squat_dtype q_dt, int64_t q_stride_batch,
                           int64_t q_stride_head, float out_scale, float* scores, int64_t s_stride_batch,
                           int64_t s_stride_head, squat_stream stream);

/* The same for a cache that holds the keys as they are BEFORE the rotary embedding (the paper's SQuat-pre
 * variant, Section 4: rotation after dequantization): cache token t is rotated to position pos0 + t before it
 * meets q (squat_key_scores_rope, or squat_key_scores_rope_per_channel for caches with key_per_channel = 1,
 * over the quantized keys; the buffered keys are rotated the same way, pairs of channels (c, c + d/2), angle
 * position * inv_freq[c]).  inv_freq: [d/2] float, device.  q is taken as given (already rotated to its own
 * position).  0 <= pos0 < 2^40. */
int squat_cache_key_scores_rope(const squat_cache* cache, const void* q, squat_dtype q_dt, int64_t q_stride_batch,
                                int64_t q_stride_head, const float* inv_freq, int64_t pos0, float out_scale,
                                float* scores, int64_t s_stride_batch, int64_t s_stride_head, squat_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* SQUAT_H */
