// Internal declarations shared by the stage executor and its gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stg {

typedef __bf16 bf16;

enum DType { DT_F32 = 0, DT_BF16 = 1 };
enum GemmMode {
  GEMM_NN = 0,  // C[m,n] = sum_k A[m*lda+k] * B[k*ldb+n]          (forward: A.W)
  GEMM_NT = 1,  // C[m,n] = sum_k A[m*lda+k] * B[n*ldb+k]          (dgrad:  dZ.W^T)
  GEMM_TN = 2   // C[m,n] = sum_k A[k*lda+m] * B[k*ldb+n]          (wgrad:  A^T.dZ)
};

struct GemmArgs {
  int mode;
  int M, N, K;
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  void* C; int64_t ldc;          // compute dtype, or fp32 when acc_f32
  const void* R; int64_t ldr;    // optional residual added in the epilogue (compute dtype), or null
  int acc_f32;                   // 1: C is fp32 and the product is added to it (C += A^T.B)
  int r_f32;                     // 1: R is fp32 (the fp32 residual stream) instead of the compute dtype
  int c_f32;                     // 1: C is stored as fp32 (no accumulate) instead of the compute dtype
  // Fused activation (forward FFN-in product only, mode GEMM_NN, no residual): besides C = z the kernel writes
  // C2 = act(z), computed from the fp32 accumulators, so the activation costs one rounding less and z is not re-read.
  int act;                       // 0 none; 1 GELU: N = f, C2[m,n] = gelu(z[m,n]); 2 SwiGLU: N = 2f (gate | up),
                                 // C2[m,j] = silu(z[m,j]) * z[m,f+j], j < f
  void* C2; int64_t ldc2;        // [M, f] in the compute dtype
  const void* bias;              // optional bias vector [N] in the compute dtype, added to every row of the product
                                 // (before the residual / activation); forward products only
  // Fused activation backward (input-gradient product of the FFN-out map only, mode GEMM_NT): the product da = dY.Wout^T
  // [M, N = f] is not stored; the kernel turns Z [M, f or 2f] (the stashed pre-activation) into dZ in place,
  // dZ = da * gelu'(z), or (SwiGLU) dgate = da * up * silu'(gate), dup = da * silu(gate).  C is unused.
  int act_bwd;                   // 0 none; 1 GELU; 2 SwiGLU
  void* Z; int64_t ldz;
};

struct AttnArgs {
  int b, s, h, hkv, hd, causal;
  const void* qkv; int64_t ld;   // [b*s, d + 2*dkv], columns q | k | v
  void* o;                       // [b*s, d]
  float* lse;                    // [b, h, s]  log-sum-exp of the scaled, masked scores
  // backward only
  const void* dout;              // [b*s, d]
  void* dqkv;                    // [b*s, d + 2*dkv]
  float* delta;                  // [b, h, s] scratch: rowsum(dout * o)
  int width;                     // workgroup shapes: 0 = chosen from the shape; forward / dQ 1 = 8 wavefronts, 2 = 4 wavefronts,
                                 // 3 = 4 wavefronts with the keys split in two; dK/dV 128 keys per workgroup for 1 and 2, 64 for 3
  float* dkv_part;               // scratch for grouped-query attention, attn_bwd_part_bytes() bytes, or null: fp32 partial
                                 // dK | dV of each split of a KV head's query heads, [nsplit][b*s][2*dkv]
};
// Into how many workgroups at most the query heads of one KV head are split in the dK/dV kernel (1 = not at all), and the
// scratch that needs.  Depends on the shape only.
int attn_bwd_splits(int b, int s, int h, int hkv);
size_t attn_bwd_part_bytes(int b, int s, int h, int hkv, int hd);

struct NormArgs {
  int kind;                      // 0 LayerNorm, 1 RMSNorm
  int rows, d;
  float eps;
  const void* x;                 // [rows, d]
  const void* gamma; const void* beta;
  void* out;                     // forward: normalised output; backward: dx (may alias x)
  float* stats;                  // [rows, 2]: mean, rstd (mean unused for RMSNorm)
  // backward only
  const void* dout;              // gradient w.r.t. the normalised output
  const void* resid;             // gradient arriving over the residual branch, added to dx
  float* dgamma; float* dbeta;   // fp32 accumulators (+=)
  float* partial;                // scratch [norm_partial_rows(), 2, d] fp32
  // storage of the residual stream: these tensors may be fp32 while the compute dtype is bf16
  int x_f32;                     // x is fp32
  int resid_f32;                 // resid is fp32
  int out_f32;                   // backward: dx is stored as fp32
  void* out_lp;                  // backward, optional: second copy of dx in the compute dtype (a GEMM operand)
};

struct ActArgs {
  int kind;                      // 0 GELU (erf), 1 SwiGLU
  int rows, f;
  void* z;                       // [rows, f] (GELU) or [rows, 2f] (gate | up); backward overwrites it with dz
  void* a;                       // forward out [rows, f]
  const void* da;                // backward in  [rows, f]
};

int norm_partial_rows();

// plain reference kernels (any dtype); one kernel per mathematical step
hipError_t gemm_ref(DType dt, const GemmArgs& g, hipStream_t s);
hipError_t attn_fwd_ref(DType dt, const AttnArgs& a, hipStream_t s);
hipError_t attn_bwd_ref(DType dt, const AttnArgs& a, hipStream_t s);

// bandwidth-bound kernels (wavefront reductions, 16-byte accesses)
hipError_t norm_fwd(DType dt, const NormArgs& n, hipStream_t s);
hipError_t norm_bwd(DType dt, const NormArgs& n, hipStream_t s);
// the same with the partial sums in a fixed device array of the library (n.partial ignored); d <= norm_bwd_noalloc_max_d()
hipError_t norm_bwd_noalloc(DType dt, const NormArgs& n, hipStream_t s);
int norm_bwd_noalloc_max_d();
hipError_t act_fwd(DType dt, const ActArgs& a, hipStream_t s);
hipError_t act_bwd(DType dt, const ActArgs& a, hipStream_t s);
// dbias[n] += sum over rows of dz[row, n] (fp32, fixed summation order); partial: bias_grad_partial_bytes(n) bytes
size_t bias_grad_partial_bytes(int n);
hipError_t bias_grad(DType dt, const void* dz, int64_t ld, int rows, int n, float* partial, float* dbias, hipStream_t s);
hipError_t fill_zero_f32(float* p, size_t n, hipStream_t s);
hipError_t copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t widen_to_f32(DType dt, float* dst, const void* src, size_t n, hipStream_t s);   // dst[i] = (float)src[i]
// rotary position embedding: table [s][hd/2] of (cos, sin) pairs; rotation in place of the first nh heads of each row
hipError_t rope_table(float* table, int s, int hd, double theta, hipStream_t st);
hipError_t rope_apply(DType dt, void* x, int64_t ld, int64_t rows, int s, int nh, int hd, const float* table, int inverse,
                      hipStream_t st);

// tuned gfx950 kernels (bf16 MFMA)
bool gemm_mfma_supported(const GemmArgs& g);
// tile_shape: 0 = full 256 x 256 tiles, half-height ones for a thin last round or a small product; 1 = full tiles only;
// 2 = half-height tiles only (1 and 2 exist so that tests reach both on any shape)
hipError_t gemm_mfma(const GemmArgs& g, hipStream_t s, int tile_shape = 0);
// several weight-gradient (TN, fp32-accumulating) products in one launch of persistent workgroups; each may reduce
// over nseg operand pairs in turn, pair s at (A + seg_delta[s] bytes, B + seg_delta[s] bytes), seg_delta[0] = 0
constexpr int GEMM_MAX_SEG = 8;
bool gemm_mfma_wgrad_group_supported(const GemmArgs* list, int n, int nseg, const int64_t* seg_delta);
hipError_t gemm_mfma_wgrad_group(const GemmArgs* list, int n, int nseg, const int64_t* seg_delta, hipStream_t s);
bool attn_mfma_supported(const AttnArgs& a);
hipError_t attn_fwd_mfma(const AttnArgs& a, hipStream_t s);
hipError_t attn_bwd_mfma(const AttnArgs& a, hipStream_t s);

// scalar conversions
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // round to nearest even

}  // namespace stg
