/* chunkflow_diag.h -- diagnostic entry points of libchunkflow.so: single kernels exposed so that each
 * can be checked against the oracle in isolation, the host-only views of two launch planners, and a
 * matrix-core rate probe.  None of them is part of the block path's contract (chunkflow.h); tests and
 * microbenchmarks use them.  Same conventions: 0 or a negative cf_status, cf_last_error(NULL) for text,
 * every pointer is DEVICE memory unless named host_*, streams are hipStream_t passed as void*.
 */
#ifndef CHUNKFLOW_DIAG_H
#define CHUNKFLOW_DIAG_H

#include "chunkflow.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Host-only view of how an attention launch over H heads, nq queries and nk keys of width head_dim is
 * shaped (Sec. 2.1: each rank attends over the whole sequence for its heads; App. B: the 4*B*S^2*d
 * term): *waves_per_workgroup receives 4 (two workgroups per CU), 7 or 8 (one), each wave owning 32
 * queries.  The choice minimises an estimate of the launch's time: generations of workgroups times the
 * time of one generation, fitted to measurements.  No GPU is touched.  CF_ERR_ARG: non-positive
 * sizes, head_dim other than 64 or 128, NULL result. */
int cf_plan_attention(int32_t H, int32_t nq, int32_t nk, int32_t head_dim, int32_t* waves_per_workgroup);

/* Host-only view of the tile a linear layer over m_rows tokens and n_features output features is
 * launched with (the GEMMs of App. B): *tile_rows receives 256 (256 x 256 tiles, one workgroup per CU)
 * or 128 (128 x 128 tiles, two per CU).  The big tile has the better arithmetic intensity; the small
 * one is taken where the big one would leave most CUs without a tile.  No GPU is touched.
 * CF_ERR_ARG: non-positive sizes, NULL result. */
int cf_plan_linear(int32_t m_rows, int32_t n_features, int32_t* tile_rows);

/* ---- single kernels.  `blob` holds W (and bias) at the given byte offsets. */
/* out[m,n] = A[m,:] . W[n,:] + bias[n]; features < n_split stored bf16 to out0[m*ld0+n], the rest
 * through GELU (tanh form, or erf form if gelu_erf) to out1[m*ld1 + n - n_split] (App. B linear layers). */
int cf_op_linear(const uint16_t* A, int32_t lda, const void* blob, uint64_t w_off, int64_t bias_off,
                 int32_t M, int32_t N, int32_t K, int32_t n0, int32_t n1, int32_t n_split,
                 uint16_t* out0, int32_t ld0, uint16_t* out1, int32_t ld1, int32_t gelu_erf, void* stream);
/* y = resid + gate * (A . W^T + bias), fp32 (gate NULL = 1). */
int cf_op_linear_residual(const uint16_t* A, int32_t lda, const void* blob, uint64_t w_off, int64_t bias_off,
                          int32_t M, int32_t N, int32_t K, const float* resid, const float* gate,
                          float* y, void* stream);
/* O[h,q,:] = softmax(Q K^T / sqrt(hd)) V; Q [H,nq,hd], K [H,nk,hd], Vt [H,hd,nk_pad] (pad zero),
 * O [H,nq,hd] (App. B attention term, no mask). */
int cf_op_attention(const uint16_t* Q, const uint16_t* K, const uint16_t* Vt, uint16_t* O,
                    int32_t H, int32_t nq, int32_t nk, int32_t nk_pad, int32_t hd, void* stream);
/* xn = LayerNorm(x) * (1 + scale) + shift, bf16 out. */
int cf_op_ln_modulate(const float* x, const float* shift, const float* scale, uint16_t* xn,
                      int32_t rows, int32_t d, void* stream);
/* m = W t + b over a blob holding W [n,K] and b [n]. */
int cf_op_modvec(const void* blob, uint64_t w_off, uint64_t b_off, const float* t, float* m,
                 int32_t n, int32_t K, void* stream);
/* Diagnostic, not part of the block path: 256 workgroups of 4 waves issue `iters` x 16 bf16 MFMAs
 * (32x32x16) each on registers alone; a launch is 256 * 4 * iters * 16 * 32768 FLOPs.  Timed by the
 * caller, it gives the matrix-core rate the chip sustains under load (Sec. 3.1's eta_c * P_peak has
 * this as its ceiling, not the published peak).  The clock the chip settles to depends on the data:
 * random_operands = 0 repeats one pair of small-valued fragments, 1 cycles through sixteen pairs of
 * unit-variance pseudo-random fragments.  `out`: 65536 floats of device memory. */
int cf_op_mfma_rate(int32_t iters, int32_t random_operands, float* out, void* stream);
/* Diagnostic, not part of the block path: the same loop with the other work a kernel's waves have to issue
 * beside their MFMAs -- per 16 MFMAs a wave makes `reads_per_16` LDS fragment reads (16 bytes per lane, through a
 * ring of four fragments) and per MFMA `valu_per_mfma` fused multiply-adds and `exp_per_mfma` exp2's; `waves`
 * (4 or 8) waves per workgroup, one workgroup per CU, no global memory traffic, no barriers.  Timed by the
 * caller it gives the ceiling of an instruction mix: the attention kernel's is one read, about four VALU
 * operations and one exp2 per MFMA on 8 waves, the GEMM's one read per two MFMAs on 4 waves.  A launch is
 * 256 * waves * iters * 16 * 32768 FLOPs.  `out`: 256 * 64 * waves floats of device memory.  Built mixes:
 * reads_per_16 in {0, 8, 16} x (valu, exp) in {(0,0)}, and (2,0), (4,0) without reads, (2,1), (4,1) with any
 * reads; anything else is CF_ERR_ARG. */
int cf_op_mix_rate(int32_t iters, int32_t waves, int32_t reads_per_16, int32_t valu_per_mfma, int32_t exp_per_mfma,
                   float* out, void* stream);
#ifdef __cplusplus
}
#endif
#endif /* CHUNKFLOW_DIAG_H */
