/*
 * tucker_convert.h -- C ABI of the weight front-ends of the MI355X (gfx950) Tucker-attention
 * library: classic attention weights in, Tucker-attention weights out, all on the device, so
 * that an MHA / GQA / MQA / MLA layer runs through the one entry point of tucker_attn.h.
 *
 * Same library (libtucker_attn.so), same conventions as tucker_attn.h: row-major contiguous
 * tensors, device pointers unless marked HOST, caller-owned buffers, a status return
 * (TUCKER_ATTN_* codes), nothing aborts or prints.  Storage type `dtype` (TUCKER_ATTN_F32 |
 * TUCKER_ATTN_BF16) applies to every weight read and written.
 *
 * Classic weights: WQ [d, nH*dH] with head i in columns i*dH .. (i+1)*dH-1 (same for WK, WV and
 * the up-projections), WO [nH*dH, d] with head i in the matching rows.
 */
#ifndef TUCKER_CONVERT_H
#define TUCKER_CONVERT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Device pointers that receive Tucker weights (shapes as in tucker_attn_weights, for the ranks
 * each call states); caller-owned, overwritten. */
typedef struct {
  void *C, *U1, *U2, *U3, *Ct, *Ut1, *Ut2, *Ut3;
} tucker_convert_weights_out;

/*
 * Grouped-query attention with nG key-value heads (nG = nH: MHA, nG = 1: MQA) as Tucker
 * attention, exactly (appendix "Tucker Representations of MQA, GQA, and MLA": the lemma on
 * D_i = A_i B_i^T and the theorem on the ranks of GQA): selector cores
 * C[i,(i,l),(g(i),l)] = 1, g(i) = i / (nH/nG), identity head factors, U2 = WQ, U3 = WK,
 * U~2 = WO^T, U~3 = WV.  Ranks of both tensors: (nH, nH*dH, nG*dH).
 *   WQ [d, nH*dH], WK, WV [d, nG*dH], WO [nH*dH, d]   in
 *   out: C, Ct [nH, nH*dH, nG*dH]; U1, Ut1 [nH, nH]; U2, Ut2 [d, nH*dH]; U3, Ut3 [d, nG*dH]
 * INVALID_ARG: null pointer, non-positive size, nH not a multiple of nG.  Enqueues on hip_stream.
 */
int tucker_convert_from_gqa(int32_t dtype, int32_t d, int32_t nH, int32_t dH, int32_t nG,
                            const void *WQ, const void *WK, const void *WV, const void *WO,
                            const tucker_convert_weights_out *out, void *hip_stream);

/*
 * Multi-head latent attention as Tucker attention, exactly (theorem on the ranks of MLA, same
 * appendix): U2 = WDQ, U3 = WDKV, core slices C[i] = WUQ_i WUK_i^T [dcQ, dcK] (products
 * accumulated in fp32, rounded once to the storage type), identity head factors; post-softmax
 * U~2 = WO^T, U~3 = WDV, core slice C~[i] = rows of head i filled with WUV_i^T, zero elsewhere.
 * With latent RoPE enabled in the layer this is the coupled-RoPE form of Section "Simplified
 * RoPE for MLA": C[i] is the fused query matrix and the rotation acts in the key latent.
 *   WDQ [d, dcQ], WUQ [dcQ, nH*dH], WDKV [d, dcK], WUK, WUV [dcK, nH*dH], WO [nH*dH, d]   in
 *   WDV [d, dcK] in, or NULL: the value latent is the key latent (run the layer with
 *   shared_kv = 1); out->Ut3 is then not written and may be NULL
 *   out: C [nH, dcQ, dcK]; Ct [nH, nH*dH, dcK]; U1, Ut1 [nH, nH]; U2 [d, dcQ]; U3, Ut3 [d, dcK];
 *        Ut2 [d, nH*dH]
 * Enqueues on hip_stream.
 */
int tucker_convert_from_mla(int32_t dtype, int32_t d, int32_t nH, int32_t dH, int32_t dcQ, int32_t dcK,
                            const void *WDQ, const void *WUQ, const void *WDKV, const void *WUK,
                            const void *WDV, const void *WUV, const void *WO,
                            const tucker_convert_weights_out *out, void *hip_stream);

/* What one tucker_convert_from_mha_hosvd call did; plain host data. */
typedef struct {
  int32_t sweeps[6];        /* Jacobi sweeps of the eigen-problems of W modes 1, 2, 3 and W~ modes 1, 2, 3    */
                            /* (0: not solved -- one head, or mode 3 of W~ with shared_kv)                    */
  int64_t jacobi_launches;  /* step kernels launched for the d x d problems (modes 2 and 3)                   */
  double  jacobi_ms;        /* time of those launches on the stream, from HIP events around each iteration    */
  double  jacobi_bytes;     /* bytes they read and wrote: every launch rotates all d rows once, 2 * 8 * d * d */
} tucker_convert_hosvd_info;

/* Bytes of device workspace tucker_convert_from_mha_hosvd needs; 0 if an argument is invalid. */
size_t tucker_convert_hosvd_workspace_bytes(int32_t d, int32_t nH, int32_t dH);

/*
 * Multi-head attention to Tucker attention of given ranks by a truncated higher-order SVD of
 * the stacked per-head products W_i = WQ_i WK_i^T and W~_i = (WV_i WO_i)^T (appendix
 * "Converting pretrained MHA parameters to approximate attention parameters").  Each factor is
 * the leading left singular vectors of a mode unfolding, computed as eigenvectors of its Gram
 * matrix (formed from the dH-wide factors, the d x d products are never built) by a one-sided
 * Jacobi iteration; the core is the tensor contracted with the transposed factors.  All
 * arithmetic in fp64; results rounded once to the storage type.  Columns are ordered by
 * decreasing singular value and signed so that the entry of largest magnitude is positive.
 *   WQ, WK, WV [d, nH*dH], WO [nH*dH, d]                       in
 *   r1 <= nH, r2 <= d, r3 <= d; rt1, rt2, rt3 alike            target ranks (pre / post softmax)
 *   shared_kv   1: the key factor U3 also serves as value factor (needs rt3 == r3); out->Ut3
 *               is not written and may be NULL
 *   out: C [r1,r2,r3], U1 [nH,r1], U2 [d,r2], U3 [d,r3], Ct [rt1,rt2,rt3], Ut1 [nH,rt1],
 *        Ut2 [d,rt2], Ut3 [d,rt3]
 *   singular_values  HOST, nullable: 2 * (nH + 2d) doubles; singular values of the mode-1, -2,
 *               -3 unfoldings of W, then of W~, each in decreasing order (with shared_kv the
 *               last d entries are zero); square roots of Gram eigenvalues, so their squares
 *               are accurate to about 1e-13 of the largest square
 *   info        HOST, nullable: iteration counts and the time of the dominant kernel
 *   workspace   device, >= tucker_convert_hosvd_workspace_bytes(d, nH, dH), 256-byte aligned
 * Unlike the other entry points this call synchronises hip_stream several times (the iteration
 * count is data dependent) and returns when the results are complete.  A requested rank beyond
 * the numerical rank of an unfolding is reported as TUCKER_ATTN_UNSUPPORTED_SHAPE after the
 * kernels have run (outputs are then undefined).  d <= 8192, nH <= 256.
 */
int tucker_convert_from_mha_hosvd(int32_t dtype, int32_t d, int32_t nH, int32_t dH,
                                  const void *WQ, const void *WK, const void *WV, const void *WO,
                                  int32_t r1, int32_t r2, int32_t r3,
                                  int32_t rt1, int32_t rt2, int32_t rt3, int32_t shared_kv,
                                  const tucker_convert_weights_out *out, double *singular_values,
                                  tucker_convert_hosvd_info *info, void *workspace, size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TUCKER_CONVERT_H */
