/*
 * stage_kernels.h -- kernel-level entry points of the stage engine.
 *
 * The same HIP kernels that stage_forward / stage_backward_input /
 * stage_backward_weight launch, callable one at a time so that each step of
 * the F / B / W path (paper section 3.1, Appendix B) can be checked against
 * its definition and timed against its roofline in isolation.
 *
 * All data pointers are DEVICE memory owned by the caller; nothing is
 * allocated, work is enqueued on `hip_stream` (hipStream_t, NULL = default
 * stream) without synchronising.  dtype / norm / act codes are the STAGE_*
 * enums of stage.h.  kernel_set: 0 = tuned gfx950 kernels where one exists for
 * the shape, 1 = plain reference HIP kernels.  stage_kernel_gemm and the
 * attention entries also take 2 and 3: the tuned kernels with a choice they
 * normally make from the shape fixed, so that tests reach both variants on any
 * shape -- GEMM: 2 = full 256 x 256 tiles only, 3 = half-height tiles only, 4 (stage_kernel_gemm, forward and
 * input-gradient layouts) = 128 x 128 tiles only;
 * attention: 2 / 3 = forward and dQ workgroups of 8 / 4 wavefronts (dK/dV workgroups of 128 keys), 4 = forward and dQ
 * workgroups of 64 queries whose two wavefronts per query block each take half of the keys, dK/dV workgroups of 64 keys.
 * Return: 0, or STAGE_E_INVAL for
 * a shape the kernel does not take, STAGE_E_HIP for a failed launch.
 */
#ifndef PAPER_2507_00217_STAGE_KERNELS_H
#define PAPER_2507_00217_STAGE_KERNELS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* mode 0 (forward,  A.W):    C[m,n] = sum_k A[m*lda+k] * B[k*ldb+n] (+ R[m*ldr+n])
 * mode 1 (dgrad,   dZ.W^T):  C[m,n] = sum_k A[m*lda+k] * B[n*ldb+k]
 * mode 2 (wgrad,   A^T.dZ):  C[m,n] += sum_k A[k*lda+m] * B[k*ldb+n], C fp32 (acc_f32 must be 1)
 * A, B, R and (unless acc_f32) C are in the compute dtype; R may be NULL. */
int stage_kernel_gemm(int dtype, int mode, int M, int N, int K, const void* A, int64_t lda, const void* B, int64_t ldb,
                      void* C, int64_t ldc, const void* R, int64_t ldr, int acc_f32, int kernel_set, void* hip_stream);

/* The forward FFN-in product with its activation (paper section 3.1: part of a chunk's F block): Z = A.B with B [K, f]
 * (GELU) or [K, 2f] (SwiGLU, columns gate | up), and Aout [M, f] = gelu(Z) or silu(Z[:, :f]) * Z[:, f:].  The tuned kernel
 * forms the activation from the fp32 accumulators in the product's epilogue (one rounding less than reading Z back, and Z
 * is not re-read); the plain kernels (kernel_set 1, or fp32) run the product and then the activation kernel on the stored
 * Z, which needs ldz = f or 2f and lda_out = f.  kernel_set 2 / 3 as for stage_kernel_gemm. */
int stage_kernel_gemm_act(int dtype, int act, int M, int f, int K, const void* A, int64_t lda, const void* B, int64_t ldb,
                          void* Z, int64_t ldz, void* Aout, int64_t lda_out, int kernel_set, void* hip_stream);

/* The input-gradient product of the FFN-out map with the activation backward (part of a chunk's B block): da = dY.W^T with
 * W [f, K] (the map's weight, [in, out]), then Z [M, f] (GELU) or [M, 2f] (SwiGLU, gate | up) is overwritten by
 * dZ = da * gelu'(Z), or dgate = da * up * silu'(gate), dup = da * silu(gate).  The tuned kernel does this in the
 * product's epilogue on the fp32 accumulators (da is never stored; da_scratch may be NULL); the plain kernels (kernel_set
 * 1, or fp32) store da [M, f] in da_scratch and run the activation kernel, which needs ldz = f or 2f. */
int stage_kernel_gemm_act_bwd(int dtype, int act, int M, int f, int K, const void* dY, int64_t ldy, const void* W, int64_t ldw,
                              void* Z, int64_t ldz, void* da_scratch, int kernel_set, void* hip_stream);

/* n weight-gradient products (mode 2 above) in one call: C_p[M_p,N_p] += A_p^T . B_p for p = 0..n-1, the separately
 * schedulable W block of the paper's Appendix B for several linear maps at once.  All array arguments are HOST arrays of
 * length n (the pointers in A, B, C are device pointers); the C_p must not overlap.  Results are bit-identical to n calls
 * of stage_kernel_gemm in mode 2.  n = 0 is a no-op; STAGE_E_INVAL for a negative n, a null array or a null entry. */
int stage_kernel_wgrad_group(int dtype, int n, const int* M, const int* N, const int* K, const void* const* A,
                             const int64_t* lda, const void* const* B, const int64_t* ldb, float* const* C,
                             const int64_t* ldc, int kernel_set, void* hip_stream);

/* Rotary position embedding.  table: [s, hd/2] pairs (cos, sin) of position * theta^(-2p/hd), built by the first call;
 * the second rotates, in place, pairs (2p, 2p+1) of the first n_heads heads of every row of x [b*s, ld] (q and k of a
 * qkv buffer: n_heads = h + hkv), or applies the transpose (inverse != 0), which is the backward pass. */
int stage_kernel_rope_table(int s, int hd, float theta, float* table, void* hip_stream);
int stage_kernel_rope(int dtype, int b, int s, int n_heads, int hd, int inverse, void* x, int64_t ld, const float* table,
                      void* hip_stream);

/* qkv: [b*s, (h + 2*hkv)*hd] rows of q | k | v;  o: [b*s, h*hd];  lse: [b, h, s] fp32. */
int stage_kernel_attention_fwd(int dtype, int b, int s, int h, int hkv, int hd, int causal, const void* qkv, void* o,
                               float* lse, int kernel_set, void* hip_stream);
/* dqkv laid out like qkv; delta: [b, h, s] fp32 scratch. */
int stage_kernel_attention_bwd(int dtype, int b, int s, int h, int hkv, int hd, int causal, const void* qkv,
                               const void* o, const float* lse, const void* dout, void* dqkv, float* delta,
                               int kernel_set, void* hip_stream);
/* The same with caller-provided scratch of at least stage_kernel_attention_bwd_scratch_bytes() bytes (16-byte aligned):
 * with grouped-query attention and few KV heads the dK/dV pass then splits each KV head's query heads over several
 * workgroups (fp32 partial sums in the scratch, added up in a fixed order), which fills the chip.  scratch == NULL, or a
 * shape that needs none (the size query returns 0), behaves like stage_kernel_attention_bwd. */
size_t stage_kernel_attention_bwd_scratch_bytes(int b, int s, int h, int hkv, int hd);
int stage_kernel_attention_bwd_ws(int dtype, int b, int s, int h, int hkv, int hd, int causal, const void* qkv,
                                  const void* o, const float* lse, const void* dout, void* dqkv, float* delta,
                                  void* scratch, size_t scratch_bytes, int kernel_set, void* hip_stream);

/* stats: [rows, 2] fp32 (mean, rstd). beta ignored for RMSNorm. */
int stage_kernel_norm_fwd(int dtype, int norm, int rows, int d, float eps, const void* x, const void* gamma,
                          const void* beta, void* out, float* stats, void* hip_stream);
/* dx = resid + norm'(dout) (resid may be NULL; dx may alias x); dgamma/dbeta fp32 += ;
 * partial: scratch of stage_kernel_norm_partial_bytes(d) bytes. */
int stage_kernel_norm_bwd(int dtype, int norm, int rows, int d, const void* x, const float* stats, const void* gamma,
                          const void* dout, const void* resid, void* dx, float* dgamma, float* dbeta, float* partial,
                          void* hip_stream);
size_t stage_kernel_norm_partial_bytes(int d);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): stage_kernel_norm_bwd without the `partial` argument.  The partial sums live in a fixed 32 MiB
 * device array inside the library (one copy per GPU, held until the process ends), which limits it to d <= 8192:
 * a wider row returns STAGE_E_INVAL with nothing enqueued.  The call allocates and frees nothing.  It acts on the
 * current device, which must be the one hip_stream and the data pointers belong to.  All calls on one GPU share the
 * array: calls that overlap on one GPU (different streams) race; calls on one stream are ordered and need no clearing
 * in between.  Same kernels, same results, bit for bit, as stage_kernel_norm_bwd. */
int stage_kernel_norm_bwd_noalloc(int dtype, int norm, int rows, int d, const void* x, const float* stats, const void* gamma,
                                  const void* dout, const void* resid, void* dx, float* dgamma, float* dbeta,
                                  void* hip_stream);

/* Gradient of a linear map's bias (layers with biases): dbias[j] += sum over rows of dz[row * ld + j], j < n, fp32, in a
 * fixed summation order.  n and ld multiples of 16 bytes' worth of elements; scratch: stage_kernel_bias_grad_scratch_bytes(n). */
size_t stage_kernel_bias_grad_scratch_bytes(int n);
int stage_kernel_bias_grad(int dtype, int rows, int n, const void* dz, int64_t ld, float* dbias, float* scratch, void* hip_stream);

/* GELU: z [rows, f]; SwiGLU: z [rows, 2f] (gate | up).  a, da: [rows, f].  Backward overwrites z with dz. */
int stage_kernel_act_fwd(int dtype, int act, int rows, int f, const void* z, void* a, void* hip_stream);
int stage_kernel_act_bwd(int dtype, int act, int rows, int f, void* z, const void* da, void* hip_stream);

/* Measurement aid (not an operation of the paper): runs nothing but back-to-back bf16 MFMAs on every compute unit for
 * `iters` (1 .. 2^22) rounds of 32 v_mfma_f32_16x16x32_bf16 per wavefront and reports the rate reached and the shader clock held meanwhile.
 * random_operands = 0 uses the constant 1.0, != 0 uniform values in [-1, 1): the clock, and with it the rate a kernel
 * can approach on real data, depends on the operands.  scratch_dev: device memory of at least 16 + 2048 * (number of
 * compute units) bytes, 16-byte aligned (1 MiB covers any gfx950 part); its contents afterwards are meaningless.
 * Allocates nothing; synchronizes hip_stream.  Returns STAGE_OK, STAGE_E_INVAL (iters out of range, null output,
 * scratch null, misaligned or too small) or STAGE_E_HIP. */
int stage_probe_mfma_ceiling(int random_operands, int iters, void* scratch_dev, size_t scratch_bytes, double* tflops,
                             double* shader_mhz, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
