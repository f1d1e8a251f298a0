// Plain reference HIP kernels: one kernel per mathematical step, fp32 arithmetic,
// any storage dtype.  They are the compute path of the fp32 configuration (whose
// shapes are launch-bound, not roofline-bound) and an A/B baseline for the tuned
// bf16 kernels.  Definitions follow the split of a linear layer's backward into
// input-gradient and weight-gradient products (paper Appendix B).
#include "common.h"

namespace stg {

// ---------------------------------------------------------------------------
// GEMM: 64x64 tile, 256 threads, 4x4 outputs per thread, K step 16
// ---------------------------------------------------------------------------
template <typename T, int MODE>
__global__ __launch_bounds__(256) void gemm_ref_kernel(GemmArgs g) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const T* A = (const T*)g.A;
  const T* B = (const T*)g.B;
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < g.K; k0 += BK) {
    for (int i = tid; i < BM * BK; i += 256) {
      int m, k;
      if (MODE == GEMM_TN) { m = i % BM; k = i / BM; } else { k = i % BK; m = i / BK; }
      int gm = m0 + m, gk = k0 + k;
      float v = 0.f;
      if (gm < g.M && gk < g.K)
        v = to_f32(MODE == GEMM_TN ? A[(int64_t)gk * g.lda + gm] : A[(int64_t)gm * g.lda + gk]);
      As[k][m] = v;
    }
    for (int i = tid; i < BN * BK; i += 256) {
      int n, k;
      if (MODE == GEMM_NT) { k = i % BK; n = i / BK; } else { n = i % BN; k = i / BN; }
      int gn = n0 + n, gk = k0 + k;
      float v = 0.f;
      if (gn < g.N && gk < g.K)
        v = to_f32(MODE == GEMM_NT ? B[(int64_t)gn * g.ldb + gk] : B[(int64_t)gk * g.ldb + gn]);
      Bs[k][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][tm + i]; b[i] = Bs[k][tn + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int gm = m0 + tm + i;
    if (gm >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tn + j;
      if (gn >= g.N) continue;
      if (g.acc_f32) {
        float* C = (float*)g.C;
        C[(int64_t)gm * g.ldc + gn] += acc[i][j];
      } else {
        float v = acc[i][j];
        if (g.bias) v += to_f32(((const T*)g.bias)[gn]);
        if (g.R) v += g.r_f32 ? ((const float*)g.R)[(int64_t)gm * g.ldr + gn] : to_f32(((const T*)g.R)[(int64_t)gm * g.ldr + gn]);
        if (g.c_f32) ((float*)g.C)[(int64_t)gm * g.ldc + gn] = v;
        else ((T*)g.C)[(int64_t)gm * g.ldc + gn] = from_f32<T>(v);
      }
    }
  }
}

template <typename T>
static hipError_t gemm_ref_t(const GemmArgs& g, hipStream_t s) {
  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64), block(256);
  switch (g.mode) {
    case GEMM_NN: hipLaunchKernelGGL((gemm_ref_kernel<T, GEMM_NN>), grid, block, 0, s, g); break;
    case GEMM_NT: hipLaunchKernelGGL((gemm_ref_kernel<T, GEMM_NT>), grid, block, 0, s, g); break;
    case GEMM_TN: hipLaunchKernelGGL((gemm_ref_kernel<T, GEMM_TN>), grid, block, 0, s, g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t gemm_ref(DType dt, const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipSuccess;
  return dt == DT_F32 ? gemm_ref_t<float>(g, s) : gemm_ref_t<bf16>(g, s);
}

// ---------------------------------------------------------------------------
// Attention, one workgroup per (sequence, query head, query position).
// Scores of the row live in LDS (4*s bytes), softmax in fp32.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float block_reduce(float v, bool is_max, float* red) {
  for (int o = 32; o > 0; o >>= 1) {
    float t = __shfl_xor(v, o, 64);
    v = is_max ? fmaxf(v, t) : v + t;
  }
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float r = red[0];
  for (int i = 1; i < nw; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
  return r;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_ref_kernel(AttnArgs a) {
  extern __shared__ float sm[];
  float* sc = sm;                 // [s]
  float* qs = sm + a.s;           // [hd]
  float* red = qs + a.hd;         // [8]
  const int i = blockIdx.x, j = blockIdx.y, ib = blockIdx.z;
  const int d = a.h * a.hd, dkv = a.hkv * a.hd, g = j / (a.h / a.hkv);
  const T* base = (const T*)a.qkv + (int64_t)ib * a.s * a.ld;
  const T* q = base + (int64_t)i * a.ld + j * a.hd;
  const T* kp = base + d + g * a.hd;
  const T* vp = base + d + dkv + g * a.hd;
  const int nk = a.causal ? i + 1 : a.s;
  const float scale = rsqrtf((float)a.hd);
  for (int t = threadIdx.x; t < a.hd; t += blockDim.x) qs[t] = to_f32(q[t]);
  __syncthreads();
  float mx = -INFINITY;
  for (int u = threadIdx.x; u < nk; u += blockDim.x) {
    const T* kr = kp + (int64_t)u * a.ld;
    float acc = 0.f;
    for (int t = 0; t < a.hd; ++t) acc = fmaf(qs[t], to_f32(kr[t]), acc);
    acc *= scale;
    sc[u] = acc;
    mx = fmaxf(mx, acc);
  }
  mx = block_reduce(mx, true, red);
  float sum = 0.f;
  for (int u = threadIdx.x; u < nk; u += blockDim.x) {
    float e = expf(sc[u] - mx);
    sc[u] = e;
    sum += e;
  }
  sum = block_reduce(sum, false, red);
  __syncthreads();
  const float inv = 1.f / sum;
  for (int t = threadIdx.x; t < a.hd; t += blockDim.x) {
    float acc = 0.f;
    for (int u = 0; u < nk; ++u) acc = fmaf(sc[u], to_f32(vp[(int64_t)u * a.ld + t]), acc);
    ((T*)a.o)[((int64_t)ib * a.s + i) * d + j * a.hd + t] = from_f32<T>(acc * inv);
  }
  if (threadIdx.x == 0) a.lse[((int64_t)ib * a.h + j) * a.s + i] = mx + logf(sum);
}

// delta[b,h,i] = sum_t dout[i,h,t] * o[i,h,t]
template <typename T>
__global__ __launch_bounds__(64) void attn_delta_ref_kernel(AttnArgs a) {
  const int i = blockIdx.x, j = blockIdx.y, ib = blockIdx.z;
  const int d = a.h * a.hd;
  const int64_t off = ((int64_t)ib * a.s + i) * d + j * a.hd;
  float acc = 0.f;
  for (int t = threadIdx.x; t < a.hd; t += 64)
    acc += to_f32(((const T*)a.dout)[off + t]) * to_f32(((const T*)a.o)[off + t]);
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (threadIdx.x == 0) a.delta[((int64_t)ib * a.h + j) * a.s + i] = acc;
}

// dq[i] = scale * sum_u ds[i,u] k[u],   ds = p * (dout.v - delta)
template <typename T>
__global__ __launch_bounds__(256) void attn_dq_ref_kernel(AttnArgs a) {
  extern __shared__ float sm[];
  float* ds = sm;                 // [s]
  float* qs = sm + a.s;           // [hd]
  float* dos = qs + a.hd;         // [hd]
  const int i = blockIdx.x, j = blockIdx.y, ib = blockIdx.z;
  const int d = a.h * a.hd, dkv = a.hkv * a.hd, g = j / (a.h / a.hkv);
  const T* base = (const T*)a.qkv + (int64_t)ib * a.s * a.ld;
  const T* kp = base + d + g * a.hd;
  const T* vp = base + d + dkv + g * a.hd;
  const int nk = a.causal ? i + 1 : a.s;
  const float scale = rsqrtf((float)a.hd);
  const int64_t row = (int64_t)ib * a.s + i;
  for (int t = threadIdx.x; t < a.hd; t += blockDim.x) {
    qs[t] = to_f32(base[(int64_t)i * a.ld + j * a.hd + t]);
    dos[t] = to_f32(((const T*)a.dout)[row * d + j * a.hd + t]);
  }
  __syncthreads();
  const float lse = a.lse[((int64_t)ib * a.h + j) * a.s + i];
  const float dl = a.delta[((int64_t)ib * a.h + j) * a.s + i];
  for (int u = threadIdx.x; u < nk; u += blockDim.x) {
    float sacc = 0.f, dp = 0.f;
    for (int t = 0; t < a.hd; ++t) {
      sacc = fmaf(qs[t], to_f32(kp[(int64_t)u * a.ld + t]), sacc);
      dp = fmaf(dos[t], to_f32(vp[(int64_t)u * a.ld + t]), dp);
    }
    ds[u] = expf(sacc * scale - lse) * (dp - dl);
  }
  __syncthreads();
  for (int t = threadIdx.x; t < a.hd; t += blockDim.x) {
    float acc = 0.f;
    for (int u = 0; u < nk; ++u) acc = fmaf(ds[u], to_f32(kp[(int64_t)u * a.ld + t]), acc);
    ((T*)a.dqkv)[row * a.ld + j * a.hd + t] = from_f32<T>(acc * scale);
  }
}

// One workgroup per (sequence, kv head, key position u): sums over the query
// heads of the group and over query positions i >= u (causal) in a fixed order.
//   dv[u] = sum p[i,u] dout[i],   dk[u] = scale * sum ds[i,u] q[i]
template <typename T>
__global__ __launch_bounds__(256) void attn_dkv_ref_kernel(AttnArgs a) {
  extern __shared__ float sm[];
  float* ps = sm;                 // [s]
  float* dss = sm + a.s;          // [s]
  float* ks = dss + a.s;          // [hd]
  float* vs = ks + a.hd;          // [hd]
  const int u = blockIdx.x, g = blockIdx.y, ib = blockIdx.z;
  const int d = a.h * a.hd, dkv = a.hkv * a.hd, grp = a.h / a.hkv;
  const T* base = (const T*)a.qkv + (int64_t)ib * a.s * a.ld;
  const float scale = rsqrtf((float)a.hd);
  for (int t = threadIdx.x; t < a.hd; t += blockDim.x) {
    ks[t] = to_f32(base[(int64_t)u * a.ld + d + g * a.hd + t]);
    vs[t] = to_f32(base[(int64_t)u * a.ld + d + dkv + g * a.hd + t]);
  }
  const int i0 = a.causal ? u : 0;
  float dk_acc = 0.f, dv_acc = 0.f;     // thread t < hd owns component t
  for (int jj = 0; jj < grp; ++jj) {
    const int j = g * grp + jj;
    __syncthreads();
    for (int i = i0 + threadIdx.x; i < a.s; i += blockDim.x) {
      const int64_t row = (int64_t)ib * a.s + i;
      const T* q = base + (int64_t)i * a.ld + j * a.hd;
      const T* dor = (const T*)a.dout + row * d + j * a.hd;
      float sacc = 0.f, dp = 0.f;
      for (int t = 0; t < a.hd; ++t) {
        sacc = fmaf(to_f32(q[t]), ks[t], sacc);
        dp = fmaf(to_f32(dor[t]), vs[t], dp);
      }
      const int64_t si = ((int64_t)ib * a.h + j) * a.s + i;
      float p = expf(sacc * scale - a.lse[si]);
      ps[i] = p;
      dss[i] = p * (dp - a.delta[si]);
    }
    __syncthreads();
    if (threadIdx.x < a.hd) {
      const int t = threadIdx.x;
      for (int i = i0; i < a.s; ++i) {
        const int64_t row = (int64_t)ib * a.s + i;
        dv_acc = fmaf(ps[i], to_f32(((const T*)a.dout)[row * d + j * a.hd + t]), dv_acc);
        dk_acc = fmaf(dss[i], to_f32(base[(int64_t)i * a.ld + j * a.hd + t]), dk_acc);
      }
    }
  }
  if (threadIdx.x < a.hd) {
    const int t = threadIdx.x;
    const int64_t row = (int64_t)ib * a.s + u;
    ((T*)a.dqkv)[row * a.ld + d + g * a.hd + t] = from_f32<T>(dk_acc * scale);
    ((T*)a.dqkv)[row * a.ld + d + dkv + g * a.hd + t] = from_f32<T>(dv_acc);
  }
}

template <typename T>
static hipError_t attn_fwd_ref_t(const AttnArgs& a, hipStream_t s) {
  dim3 grid(a.s, a.h, a.b);
  size_t sm = (size_t)(a.s + a.hd + 8) * sizeof(float);
  hipLaunchKernelGGL((attn_fwd_ref_kernel<T>), grid, dim3(256), sm, s, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t attn_bwd_ref_t(const AttnArgs& a, hipStream_t s) {
  hipLaunchKernelGGL((attn_delta_ref_kernel<T>), dim3(a.s, a.h, a.b), dim3(64), 0, s, a);
  hipLaunchKernelGGL((attn_dq_ref_kernel<T>), dim3(a.s, a.h, a.b), dim3(256),
                     (size_t)(a.s + 2 * a.hd) * sizeof(float), s, a);
  hipLaunchKernelGGL((attn_dkv_ref_kernel<T>), dim3(a.s, a.hkv, a.b), dim3(256),
                     (size_t)(2 * a.s + 2 * a.hd) * sizeof(float), s, a);
  return hipGetLastError();
}

hipError_t attn_fwd_ref(DType dt, const AttnArgs& a, hipStream_t s) {
  return dt == DT_F32 ? attn_fwd_ref_t<float>(a, s) : attn_fwd_ref_t<bf16>(a, s);
}
hipError_t attn_bwd_ref(DType dt, const AttnArgs& a, hipStream_t s) {
  return dt == DT_F32 ? attn_bwd_ref_t<float>(a, s) : attn_bwd_ref_t<bf16>(a, s);
}

}  // namespace stg
