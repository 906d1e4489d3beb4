/*
 * tucker_attn.h -- C ABI of the MI355X (gfx950) Tucker-attention forward library.
 *
 * The layer (paper, Definition "Tucker Attention"): the pre-softmax tensor
 * W = C x1 U1 x2 U2 x3 U3 and the post-softmax tensor W~ = C~ x1 U~1 x2 U~2 x3 U~3
 * (modes: head, query/output, key/value) define, for a sequence X [N, d],
 *
 *     Y[j,k] = sum_i sum_l softmax_l( (X W_i X^T)[j,l] / sqrt(d_head) ) * (W~_i X^T)[k,l]
 *
 * (Section "Tensor attention reformulation", the contraction of H1 and H2 over heads
 * and sequence).  The library evaluates it in the factored order of Sections "KV
 * Caching", "Rotary Position Embedding" and "Flash Attention": shared latent
 * Qlat = X U2, K = X U3, V = X U~3; per-head queries Qhat_i = Qlat (C x1 U1)_i; latent
 * RoPE on Qhat_i and K in the r3-wide key space; online-softmax attention in which one
 * K/V pair serves all heads; head merge through (C~ x1 U~1)_i; output Y = Z U~2^T.
 *
 * Conventions
 *   - All tensors are row-major and contiguous, last index fastest.
 *   - "device" pointers are HIP device memory of the GPU that was current at
 *     tucker_attn_create; "host" pointers are ordinary process memory.
 *   - The caller owns every buffer it passes (inputs, outputs, caches, workspace); the
 *     library keeps no pointer after a call returns (one documented exception:
 *     tucker_attn_prepare_weights).  The context owns only host state
 *     and one device table of rotation cosines/sines allocated in create.
 *   - forward/decode only enqueue work on the given HIP stream and return; results are
 *     valid once the caller has synchronised that stream.  Calls that share a
 *     workspace must be ordered on one stream.
 *   - Every entry point returns a status (0 = OK, negative = error); nothing aborts,
 *     throws or prints.  Arguments and shapes are checked before anything is enqueued: on
 *     INVALID_ARG, UNSUPPORTED_SHAPE and WORKSPACE_TOO_SMALL no kernel has been launched.
 *     HIP_ERROR reports a failed runtime call; kernels of the same call launched before it
 *     may already be enqueued, and the outputs are then undefined.
 *   - Readings of the paper where it is silent: softmax scale 1/sqrt(d_head) with d_head a
 *     free parameter; causal = key n visible to query m iff n <= m; RoPE = rotations of
 *     adjacent channel pairs (2j,2j+1) by angle position * base^(-2j/r3), applied as
 *     x'_{2j} = x_{2j} cos - x_{2j+1} sin, x'_{2j+1} = x_{2j} sin + x_{2j+1} cos, to Qhat_i
 *     (after the core) and to K, never to V; the cache stores rotated K and plain V; a
 *     decoded token is the last row of the cache.
 */
#ifndef TUCKER_ATTN_H
#define TUCKER_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tucker_attn_ctx tucker_attn_ctx;   /* opaque */

enum { TUCKER_ATTN_F32 = 0, TUCKER_ATTN_BF16 = 1 };

enum {
  TUCKER_ATTN_OK = 0,
  TUCKER_ATTN_INVALID_ARG = -1,          /* null pointer, non-positive size, kv_len out of range ... */
  TUCKER_ATTN_UNSUPPORTED_SHAPE = -2,    /* a shape outside the limits listed at tucker_attn_create  */
  TUCKER_ATTN_WORKSPACE_TOO_SMALL = -3,
  TUCKER_ATTN_HIP_ERROR = -4             /* a HIP runtime call failed (allocation, launch)           */
};

/* Problem description; plain data, copied by create. */
typedef struct {
  int32_t d_model;        /* d: width of X and Y                                                   */
  int32_t n_heads;        /* nH                                                                    */
  int32_t d_head;         /* enters only as the softmax scale 1/sqrt(d_head)                       */
  int32_t r1, r2, r3;     /* pre-softmax Tucker ranks: head, query, key                            */
  int32_t rt1, rt2, rt3;  /* post-softmax Tucker ranks: head, output, value                        */
  int32_t causal;         /* 0 | 1                                                                 */
  int32_t use_rope;       /* 0 | 1: latent RoPE over r3 (Definition "Latent RoPE")                 */
  float   rope_base;      /* e.g. 1e4                                                              */
  int32_t dtype;          /* TUCKER_ATTN_F32 | TUCKER_ATTN_BF16: storage of X, weights, caches, Y; */
                          /* products accumulate in fp32 in both cases                             */
  int32_t max_positions;  /* rotation table covers positions 0 .. max_positions-1 (>= pos0+N, Lmax)*/
                          /* The only size the context fixes: batch and sequence length are given  */
                          /* per call and bound the workspace, which the caller sizes per call     */
                          /* with tucker_attn_workspace_bytes(ctx, B, N).                          */
  int32_t shared_kv;      /* 0 | 1: shared key-value down-projection (Section "KV Caching"): the  */
                          /* value basis IS the key basis U3, so V = X U3 is the unrotated key     */
                          /* latent; needs rt3 == r3; weights.Ut3 is ignored (may be NULL); ONE    */
                          /* cache [B, Lmax, r3] holds the UNROTATED latent and keys are rotated   */
                          /* when a cache tile is read                                             */
  int32_t save_for_backward; /* 0 | 1: training.  tucker_attn_forward then also leaves what the    */
                          /* backward pass needs (log-sum-exp of every query and head, value rows, */
                          /* transposed keys) in its workspace, and tucker_attn_workspace_bytes     */
                          /* returns the size of the backward workspace, so that one buffer serves  */
                          /* a forward call and the backward call that follows it                   */
} tucker_attn_config;

/* Device pointers to the weights; read-only, caller-owned. */
typedef struct {
  const void *C;    /* [r1, r2, r3]    pre-softmax core                 */
  const void *U1;   /* [nH, r1]        head-mode basis                  */
  const void *U2;   /* [d,  r2]        query-mode basis                 */
  const void *U3;   /* [d,  r3]        key-mode basis                   */
  const void *Ct;   /* [rt1, rt2, rt3] post-softmax core                */
  const void *Ut1;  /* [nH, rt1]       head-mode basis (post)           */
  const void *Ut2;  /* [d,  rt2]       output-mode basis                */
  const void *Ut3;  /* [d,  rt3]       value-mode basis                 */
} tucker_attn_weights;

/*
 * Create a context (Definition "Tucker Attention" fixes the shapes).  Host work plus one
 * device allocation (rotation table: for every position below max_positions the cos/sin pairs
 * of the r3/2 channel pairs, padded to a multiple of 16 pairs, fp32, built in double precision).  Limits of this build, reported as TUCKER_ATTN_UNSUPPORTED_SHAPE:
 * r3, rt3 <= 128; r2, rt2 <= 512; r1, rt1 <= 64; d_model a multiple of 8; r3 even when
 * use_rope; ranks need not be multiples of 32 (they are zero-padded internally).
 */
int tucker_attn_create(const tucker_attn_config *cfg, tucker_attn_ctx **out);

/*
 * Memory footprint of the layer (table "Comparison of the memory footprint of MHA, MQA, GQA, MLA and
 * Tucker Attention"), host arithmetic only.
 *   tucker_attn_parameter_count   number of weights of one layer: the two cores, the two head factors and
 *                                 the query / key / output / value factors, nH r1 + d (r2 + r3) + r1 r2 r3 for
 *                                 the pre-softmax tensor plus the same with the post-softmax ranks; with
 *                                 shared_kv the value factor is not counted (it is the key factor).  0 if
 *                                 cfg is NULL.
 *   tucker_attn_cache_bytes       bytes of latent KV cache the caller allocates for B sequences of up to
 *                                 Lmax tokens: B * Lmax * (r3 + rt3) elements of the storage type, B * Lmax * r3
 *                                 with shared_kv.  0 if an argument is invalid.
 */
size_t tucker_attn_parameter_count(const tucker_attn_config *cfg);
size_t tucker_attn_cache_bytes(const tucker_attn_ctx *ctx, int32_t B, int32_t Lmax);

/* Free the context and its rotation table.  NULL is ignored. */
void tucker_attn_destroy(tucker_attn_ctx *ctx);

/* Bytes of device workspace tucker_attn_forward needs for a batch of B sequences of N
 * tokens (with save_for_backward: what tucker_attn_backward needs); 0 if an argument is invalid. */
size_t tucker_attn_workspace_bytes(const tucker_attn_ctx *ctx, int32_t B, int32_t N);

/* Bytes of device workspace tucker_attn_decode needs for B sequences (it grows with B up to 32
 * sequences, the size of one pass of the decode kernels, and stays there); 0 if invalid. */
size_t tucker_attn_decode_workspace_bytes(const tucker_attn_ctx *ctx, int32_t B);

/*
 * Prefill / training-style forward of B independent sequences of N tokens at positions
 * pos0 .. pos0+N-1 (the whole path: head-mixed cores, factor projection, latent RoPE,
 * online-softmax attention, head merge, output projection).
 *   X            device [B, N, d]      in
 *   Y            device [B, N, d]      out
 *   Kcache_out   device [B, Lmax, r3]  out, nullable: rows pos0..pos0+N-1 receive the rotated keys
 *   Vcache_out   device [B, Lmax, rt3] out, nullable: same rows receive the values
 *                (both or neither; needs pos0+N <= Lmax).  With shared_kv: Vcache_out must be
 *                NULL and Kcache_out, if given, receives the UNROTATED latent rows.
 *   workspace    device, >= tucker_attn_workspace_bytes(ctx,B,N) bytes, 256-byte aligned; scratch
 *   hip_stream   a hipStream_t (NULL = the null stream)
 * Limits: B <= 65535 and B * roundup(N, 64) <= 65535 * 32 = 2 097 120 padded tokens (the launch grids),
 * reported as TUCKER_ATTN_UNSUPPORTED_SHAPE before anything is enqueued.
 */
int tucker_attn_forward(tucker_attn_ctx *ctx, const tucker_attn_weights *w,
                        const void *X, void *Y, int32_t B, int32_t N, int32_t pos0,
                        void *Kcache_out, void *Vcache_out, int32_t Lmax,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * One new token per sequence against the latent KV cache (Section "KV Caching").
 *   x        device [B, d]            in: the new token of each sequence
 *   y        device [B, d]            out
 *   Kcache   device [B, Lmax, r3]     in/out: row kv_len[b]-1 is written (rotated key of x[b])
 *   Vcache   device [B, Lmax, rt3]    in/out: row kv_len[b]-1 is written (value of x[b])
 *            With shared_kv: Vcache must be NULL and Kcache is the one cache of unrotated latent
 *            rows (row kv_len[b]-1 is written unrotated).
 *   kv_len   HOST   [B] int32         cache length INCLUDING the new token, 1 <= kv_len[b] <= Lmax;
 *                                     the query sits at position kv_len[b]-1 and attends rows 0..kv_len[b]-1
 *   B        >= 1; batches above 32 sequences run as consecutive passes of 32 on the stream
 * causal in the config is irrelevant here (the query is the last position).
 * Limits (TUCKER_ATTN_UNSUPPORTED_SHAPE): n_heads <= 64; cache rows a multiple of 16 bytes; the attended
 * part of one sequence's cache, kv_len[b] * max(r3, rt3) elements, below 2 GiB.
 */
int tucker_attn_decode(tucker_attn_ctx *ctx, const tucker_attn_weights *w,
                       const void *x, void *y, void *Kcache, void *Vcache, int32_t Lmax,
                       const int32_t *kv_len, int32_t B,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * tucker_attn_decode for callers that cannot allocate device memory or keep a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels
 * and results as tucker_attn_decode, without the workspace: the scratch memory is a 32 MiB
 * (33 554 432 bytes) device array that is part of the loaded library (each GPU the library runs on
 * holds its own copy until the process ends).  The call allocates and frees nothing.
 *   - TUCKER_ATTN_WORKSPACE_TOO_SMALL if tucker_attn_decode_workspace_bytes(ctx, B) exceeds 32 MiB
 *     (the LLaMA-7B layer shape with ranks [8,128,128] needs at most 11.1 MiB, whatever B); nothing is enqueued.
 *   - Every call on a GPU, from any context, uses that GPU's one array: calls must be ordered on one
 *     stream or otherwise synchronised; calls that overlap on one GPU race.  The array keeps the last
 *     call's contents; no part of it has to start at zero (every piece is written before it is read
 *     within a call), so nothing is cleared.
 */
int tucker_attn_decode_static(tucker_attn_ctx *ctx, const tucker_attn_weights *w,
                              const void *x, void *y, void *Kcache, void *Vcache, int32_t Lmax,
                              const int32_t *kv_len, int32_t B, void *hip_stream);

/* Device pointers that receive the weight gradients, fp32 whatever the storage type (they are
 * sums over all tokens); caller-owned, overwritten (not accumulated into). */
typedef struct {
  float *dC;    /* [r1, r2, r3]    */
  float *dU1;   /* [nH, r1]        */
  float *dU2;   /* [d,  r2]        */
  float *dU3;   /* [d,  r3]        with shared_kv: key path plus value path */
  float *dCt;   /* [rt1, rt2, rt3] */
  float *dUt1;  /* [nH, rt1]       */
  float *dUt2;  /* [d,  rt2]       */
  float *dUt3;  /* [d,  rt3]       must be NULL with shared_kv (no such weight) */
} tucker_attn_grads;

/* Bytes of device workspace tucker_attn_backward needs; 0 if an argument is invalid. */
size_t tucker_attn_backward_workspace_bytes(const tucker_attn_ctx *ctx, int32_t B, int32_t N);

/*
 * Gradients of the prefill forward (the paper trains the layer -- Section "Experiments" -- and
 * times a backward pass; the gradient is the derivative of the forward of Definition "Tucker
 * Attention" with latent RoPE, evaluated flash-style: attention probabilities are recomputed
 * from a saved log-sum-exp, never stored).  For loss = sum(dY * Y):
 *   X    device [B, N, d]   in: the forward input
 *   dY   device [B, N, d]   in: upstream gradient, storage type
 *   dX   device [B, N, d]   out: gradient of X, storage type
 *   grads                   out: gradients of the eight weight arrays (seven with shared_kv), fp32
 *   forward_state  0: the call is self-contained; it re-runs the forward up to the head merge inside
 *                  its own workspace, then the backward kernels.
 *                  1: the workspace is the one a tucker_attn_forward call of this context (created
 *                  with save_for_backward = 1) just used with the same w, X, B, N and pos0, and nothing
 *                  has written to it since: the forward is not run again.  INVALID_ARG if the context
 *                  was created without save_for_backward.
 * Same shape limits as forward.
 * Accuracy against an fp64 chain rule on the same stored inputs: relative L2 error of every returned array at most
 * 1e-5 with fp32 storage and 2e-2 with bf16 storage.  Exception, bf16 storage: dU1 and dUt1 are a few numbers, each
 * a sum of signed terms <dG_i, C[a]>; the storage roundings of the pipeline (about 2^-9 per term) reach them
 * multiplied by the sum's cancellation factor kappa = |sum of absolute terms| / |sum|, and their error bound is
 * max(2e-2, 2^-10 kappa) (head rank 1, or a single head, gives kappa of 70 and more).
 */
int tucker_attn_backward(tucker_attn_ctx *ctx, const tucker_attn_weights *w,
                         const void *X, const void *dY, void *dX, const tucker_attn_grads *grads,
                         int32_t B, int32_t N, int32_t pos0, int32_t forward_state,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Weights that stay fixed over many calls (serving): prepare their operand-layout copies once
 * (the head-mixed cores G_i = sum_a U1[i,a] C[a] of Section "KV Caching" and the transposed, padded
 * factor matrices, step one of every forward / decode call) into a caller-owned device buffer, and
 * every later forward / decode / backward call of this context skips that step.
 *   prepared   device, >= tucker_attn_prepared_weights_bytes(ctx) bytes, 256-byte aligned
 * Exception to the ownership rule above: the context keeps the pointer `prepared` and the eight
 * weight pointers of `w` until tucker_attn_release_weights or tucker_attn_destroy; the caller keeps
 * the buffer alive and unmodified, orders the prepare call before the calls that use it (same
 * stream, or synchronised), and passes the same weight pointers to those calls (others are refused
 * with TUCKER_ATTN_INVALID_ARG).  After the weights' values change, prepare again or release.
 */
size_t tucker_attn_prepared_weights_bytes(const tucker_attn_ctx *ctx);
int tucker_attn_prepare_weights(tucker_attn_ctx *ctx, const tucker_attn_weights *w,
                                void *prepared, size_t prepared_bytes, void *hip_stream);
int tucker_attn_release_weights(tucker_attn_ctx *ctx);

/*
 * Optional per-kernel timing for benchmarks.  While enabled, forward/backward/decode bracket every
 * kernel they launch with HIP events recorded on the caller's stream; tucker_attn_profile_read
 * synchronises those events and returns, for the LAST call, the kernel count and for each
 * kernel its name and duration (the time between the two events around the launch, which includes
 * the dispatch on either side).  For the attention launch of a forward or decode call one more entry
 * follows the kernels: "attention_kernel" / "decode_attention_kernel", the duration of that kernel
 * alone, from a start and a stop event attached to its dispatch.  Event recording perturbs
 * end-to-end time slightly, so throughput is measured with profiling disabled.
 *   names   host array of n_max pointers, receives static strings (nullable)
 *   ms      host array of n_max floats (nullable)
 * Returns the number of entries of the last call (<= 41) or a negative status.
 */
int tucker_attn_profile_enable(tucker_attn_ctx *ctx, int32_t on);
int tucker_attn_profile_read(tucker_attn_ctx *ctx, const char **names, float *ms, int32_t n_max);

/*
 * Measurement aid, not part of the layer: the rate the matrix pipe of the current device sustains on a loop of
 * bf16 32x32x16 MFMAs with pseudo-random operands, eight waves on every compute unit, on the null stream (the
 * call synchronises; best of five launches).  Reports that quote a fraction of the published bf16 peak give this
 * figure beside it (the published peak assumes the maximum clock, which a board at its power limit does not hold).
 *   from_lds    0: both operands stay in registers; 1: one 2 KB operand fragment is re-read from LDS for every
 *               pair of MFMAs, the way the attention kernel is fed
 *   iters       loop length per wave (8 MFMAs each), e.g. 20000
 *   tflops_out  host, receives TFLOP/s
 */
int tucker_attn_measure_mfma_ceiling(int32_t from_lds, int32_t iters, float *tflops_out);

/* Static, human-readable text for a status code. */
const char *tucker_attn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TUCKER_ATTN_H */
