// Bandwidth-bound kernels of the stage: LayerNorm / RMSNorm forward and backward
// (wavefront reductions, rows held in registers so HBM is read once), GELU /
// SwiGLU forward and backward, fill and copy.  All accesses are 16-byte vectors.
// Norm-parameter gradients are produced here, at B time, through per-workgroup
// partial sums reduced in a fixed order (no atomics), so results do not depend
// on scheduling.
#include "common.h"

#include <mutex>

namespace stg {

template <typename T> struct Vec {
  static constexpr int N = 16 / sizeof(T);
  union { uint4 raw; T v[16 / sizeof(T)]; };
};

template <typename T> __device__ __forceinline__ Vec<T> ldv(const T* p) {
  Vec<T> r; r.raw = *reinterpret_cast<const uint4*>(p); return r;
}
template <typename T> __device__ __forceinline__ void stv(T* p, const Vec<T>& r) {
  *reinterpret_cast<uint4*>(p) = r.raw;
}

// V consecutive elements starting at element offset `off` of a row that is stored either in T or (wide) in fp32
template <typename T>
__device__ __forceinline__ void ld_row(float (&dst)[Vec<T>::N], const void* base, int64_t off, bool wide) {
  constexpr int V = Vec<T>::N;
  if (wide && sizeof(T) != 4) {
    const float4* p = reinterpret_cast<const float4*>((const float*)base + off);
#pragma unroll
    for (int q = 0; q < V / 4; ++q) { float4 t = p[q]; dst[4 * q] = t.x; dst[4 * q + 1] = t.y; dst[4 * q + 2] = t.z; dst[4 * q + 3] = t.w; }
  } else {
    Vec<T> t = ldv((const T*)base + off);
#pragma unroll
    for (int e = 0; e < V; ++e) dst[e] = to_f32(t.v[e]);
  }
}
template <typename T>
__device__ __forceinline__ void st_row(void* base, int64_t off, const float (&src)[Vec<T>::N], bool wide) {
  constexpr int V = Vec<T>::N;
  if (wide && sizeof(T) != 4) {
    float4* p = reinterpret_cast<float4*>((float*)base + off);
#pragma unroll
    for (int q = 0; q < V / 4; ++q) p[q] = make_float4(src[4 * q], src[4 * q + 1], src[4 * q + 2], src[4 * q + 3]);
  } else {
    Vec<T> o;
#pragma unroll
    for (int e = 0; e < V; ++e) o.v[e] = from_f32<T>(src[e]);
    stv((T*)base + off, o);
  }
}

constexpr int NORM_THREADS = 256;
constexpr int NORM_MAXCH = 4;          // 16-byte chunks per thread: d <= 256*4*(16/sizeof(T))
constexpr int NORM_PARTIAL_ROWS = 512;   // multiple of 4; two workgroups per CU keep more rows in flight
int norm_partial_rows() { return NORM_PARTIAL_ROWS; }

__device__ __forceinline__ float wg_sum(float v, float* red) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// out = (x - mean) * rstd * gamma + beta   |   out = x * rstd * gamma
template <typename T, int KIND>
__global__ __launch_bounds__(NORM_THREADS) void norm_fwd_kernel(NormArgs n) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[4];
  const int row = blockIdx.x;
  const int64_t roff = (int64_t)row * n.d;
  T* out = (T*)n.out + roff;
  const int nvec = n.d / V;
  float xv[NORM_MAXCH][V];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NORM_MAXCH; ++c) {
    const int vi = threadIdx.x + c * NORM_THREADS;
    if (vi < nvec) {
      ld_row<T>(xv[c], n.x, roff + vi * V, n.x_f32);
#pragma unroll
      for (int e = 0; e < V; ++e) s += (KIND == 0) ? xv[c][e] : xv[c][e] * xv[c][e];
    }
  }
  float mean = 0.f, rstd;
  const float inv_d = 1.f / (float)n.d;
  if (KIND == 0) {
    mean = wg_sum(s, red) * inv_d;
    float q = 0.f;
#pragma unroll
    for (int c = 0; c < NORM_MAXCH; ++c)
      if (threadIdx.x + c * NORM_THREADS < nvec)
#pragma unroll
        for (int e = 0; e < V; ++e) { float t = xv[c][e] - mean; q += t * t; }
    rstd = rsqrtf(wg_sum(q, red) * inv_d + n.eps);
  } else {
    rstd = rsqrtf(wg_sum(s, red) * inv_d + n.eps);
  }
  if (threadIdx.x == 0) { n.stats[2 * row] = mean; n.stats[2 * row + 1] = rstd; }
#pragma unroll
  for (int c = 0; c < NORM_MAXCH; ++c) {
    const int vi = threadIdx.x + c * NORM_THREADS;
    if (vi < nvec) {
      Vec<T> g = ldv((const T*)n.gamma + vi * V), b, o;
      if (KIND == 0) b = ldv((const T*)n.beta + vi * V);
#pragma unroll
      for (int e = 0; e < V; ++e) {
        float y = (xv[c][e] - mean) * rstd * to_f32(g.v[e]);
        if (KIND == 0) y += to_f32(b.v[e]);
        o.v[e] = from_f32<T>(y);
      }
      stv(out + vi * V, o);
    }
  }
}

// dx = resid + rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)),  dxhat = dout * gamma
// (the mean(dxhat) term is absent for RMSNorm); per-workgroup partial sums of
// dgamma = sum_rows dout * xhat and dbeta = sum_rows dout go to n.partial.
template <typename T, int KIND>
__global__ __launch_bounds__(NORM_THREADS) void norm_bwd_kernel(NormArgs n) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[4];
  const int nvec = n.d / V;
  float gam[NORM_MAXCH][V], dg[NORM_MAXCH][V], db[NORM_MAXCH][V];
#pragma unroll
  for (int c = 0; c < NORM_MAXCH; ++c) {
    const int vi = threadIdx.x + c * NORM_THREADS;
    Vec<T> g;
    if (vi < nvec) g = ldv((const T*)n.gamma + vi * V);
#pragma unroll
    for (int e = 0; e < V; ++e) { gam[c][e] = vi < nvec ? to_f32(g.v[e]) : 0.f; dg[c][e] = 0.f; db[c][e] = 0.f; }
  }
  const float inv_d = 1.f / (float)n.d;
  for (int row = blockIdx.x; row < n.rows; row += gridDim.x) {
    const int64_t roff = (int64_t)row * n.d;
    const T* dout = (const T*)n.dout + roff;
    const float mean = n.stats[2 * row], rstd = n.stats[2 * row + 1];
    float xh[NORM_MAXCH][V], dxh[NORM_MAXCH][V], res[NORM_MAXCH][V];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NORM_MAXCH; ++c) {
      const int vi = threadIdx.x + c * NORM_THREADS;
      if (vi < nvec) {
        float tx[V];
        ld_row<T>(tx, n.x, roff + vi * V, n.x_f32);
        Vec<T> td = ldv(dout + vi * V);
        if (n.resid) ld_row<T>(res[c], n.resid, roff + vi * V, n.resid_f32);     // in flight during the row reductions
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const float xhat = (tx[e] - mean) * rstd;
          const float dv = to_f32(td.v[e]);
          xh[c][e] = xhat;
          dxh[c][e] = dv * gam[c][e];
          dg[c][e] += dv * xhat;
          if (KIND == 0) db[c][e] += dv;
          s1 += dxh[c][e];
          s2 += dxh[c][e] * xhat;
        }
      }
    }
    float m1 = 0.f;
    if (KIND == 0) m1 = wg_sum(s1, red) * inv_d;
    const float m2 = wg_sum(s2, red) * inv_d;
#pragma unroll
    for (int c = 0; c < NORM_MAXCH; ++c) {
      const int vi = threadIdx.x + c * NORM_THREADS;
      if (vi < nvec) {
        float o[V];
#pragma unroll
        for (int e = 0; e < V; ++e) {
          float v = (dxh[c][e] - m1 - xh[c][e] * m2) * rstd;
          if (n.resid) v += res[c][e];
          o[e] = v;
        }
        st_row<T>(n.out, roff + vi * V, o, n.out_f32);
        if (n.out_lp) st_row<T>(n.out_lp, roff + vi * V, o, false);
      }
    }
  }
  float* pg = n.partial + (int64_t)blockIdx.x * 2 * n.d;
  float* pb = pg + n.d;
#pragma unroll
  for (int c = 0; c < NORM_MAXCH; ++c) {
    const int vi = threadIdx.x + c * NORM_THREADS;
    if (vi < nvec)
#pragma unroll
      for (int e = 0; e < V; ++e) {
        pg[vi * V + e] = dg[c][e];
        if (KIND == 0) pb[vi * V + e] = db[c][e];
      }
  }
}

// grads += sum over workgroup partials, in a fixed order: 64 columns per workgroup, FIN_WAVES wavefronts each summing
// an equal share of the partial rows (coalesced 256-byte reads, all of a wavefront's loads in flight at once: the kernel
// is a few microseconds of memory latency, not bandwidth), then wavefront 0 adds the shares in order
constexpr int FIN_WAVES = 16;
static_assert(NORM_PARTIAL_ROWS % FIN_WAVES == 0, "equal shares");
template <int KIND>
__global__ __launch_bounds__(FIN_WAVES * 64) void norm_bwd_finalize_kernel(NormArgs n, int nparts) {
  __shared__ float sg[FIN_WAVES][64], sb[FIN_WAVES][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + lane;
  float g = 0.f, b = 0.f;
  if (col < n.d) {
    constexpr int PER = NORM_PARTIAL_ROWS / FIN_WAVES;
    const float* p0 = n.partial + (int64_t)w * PER * 2 * n.d + col;
    float vg[PER], vb[PER];
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      vg[p] = p0[(int64_t)p * 2 * n.d];
      if (KIND == 0) vb[p] = p0[(int64_t)p * 2 * n.d + n.d];
    }
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      g += vg[p];
      if (KIND == 0) b += vb[p];
    }
  }
  sg[w][lane] = g; sb[w][lane] = b;
  __syncthreads();
  if (w == 0 && col < n.d) {
    float tg = sg[0][lane], tb = sb[0][lane];
#pragma unroll
    for (int k = 1; k < FIN_WAVES; ++k) { tg += sg[k][lane]; tb += sb[k][lane]; }
    n.dgamma[col] += tg;
    if (KIND == 0) n.dbeta[col] += tb;
  }
}

template <typename T>
static bool norm_shape_ok(const NormArgs& n) {
  constexpr int V = 16 / sizeof(T);
  return n.d % V == 0 && n.d / V <= NORM_THREADS * NORM_MAXCH && n.rows > 0;
}

template <typename T>
static hipError_t norm_fwd_t(const NormArgs& n, hipStream_t s) {
  if (!norm_shape_ok<T>(n)) return hipErrorInvalidValue;
  if (n.kind == 0) hipLaunchKernelGGL((norm_fwd_kernel<T, 0>), dim3(n.rows), dim3(NORM_THREADS), 0, s, n);
  else hipLaunchKernelGGL((norm_fwd_kernel<T, 1>), dim3(n.rows), dim3(NORM_THREADS), 0, s, n);
  return hipGetLastError();
}

template <typename T>
static hipError_t norm_bwd_t(const NormArgs& n, hipStream_t s) {
  if (!norm_shape_ok<T>(n)) return hipErrorInvalidValue;
  const int parts = NORM_PARTIAL_ROWS;
  const int fb = (n.d + 63) / 64;
  if (n.kind == 0) {
    hipLaunchKernelGGL((norm_bwd_kernel<T, 0>), dim3(parts), dim3(NORM_THREADS), 0, s, n);
    hipLaunchKernelGGL((norm_bwd_finalize_kernel<0>), dim3(fb), dim3(FIN_WAVES * 64), 0, s, n, parts);
  } else {
    hipLaunchKernelGGL((norm_bwd_kernel<T, 1>), dim3(parts), dim3(NORM_THREADS), 0, s, n);
    hipLaunchKernelGGL((norm_bwd_finalize_kernel<1>), dim3(fb), dim3(FIN_WAVES * 64), 0, s, n, parts);
  }
  return hipGetLastError();
}

hipError_t norm_fwd(DType dt, const NormArgs& n, hipStream_t s) {
  return dt == DT_F32 ? norm_fwd_t<float>(n, s) : norm_fwd_t<bf16>(n, s);
}
hipError_t norm_bwd(DType dt, const NormArgs& n, hipStream_t s) {
  return dt == DT_F32 ? norm_bwd_t<float>(n, s) : norm_bwd_t<bf16>(n, s);
}

// Norm backward for callers that cannot allocate device memory: the per-workgroup partial sums of dgamma / dbeta go to
// a fixed array in the library's own device image instead of a caller-provided buffer.  Every GPU the library runs on
// holds its own copy of the array, at its own address, until the process ends; `scratch` in host code is only a handle
// to the symbol, so the device address is looked up once per device and that pointer is what the kernels are given.
// The kernels write every partial they later read, so nothing has to be cleared between calls; two calls that
// overlap on one GPU (different streams) would race on the array.
constexpr int NOALLOC_MAX_D = 8192;
constexpr int NOALLOC_MAX_DEVICES = 64;
static __device__ __align__(256) float scratch[(size_t)NORM_PARTIAL_ROWS * 2 * NOALLOC_MAX_D];   // 32 MiB

int norm_bwd_noalloc_max_d() { return NOALLOC_MAX_D; }

hipError_t norm_bwd_noalloc(DType dt, const NormArgs& n, hipStream_t s) {
  static std::mutex mu;
  static float* scratch_of[NOALLOC_MAX_DEVICES] = {};
  if (n.d < 1 || n.d > NOALLOC_MAX_D) return hipErrorInvalidValue;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return hipErrorInvalidDevice;
  float* ptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!scratch_of[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));     // the current device's copy
      if (e != hipSuccess) return e;
      if (!p) return hipErrorInvalidSymbol;
      scratch_of[dev] = (float*)p;
    }
    ptr = scratch_of[dev];
  }
  NormArgs m = n;
  m.partial = ptr;
  return norm_bwd(dt, m, s);
}

// ---------------------------------------------------------------------------
// Gradient of a linear map's bias: the column sums of its dZ, added to the fp32 accumulator.  Two steps with a fixed
// summation order (no atomics): BIAS_PARTS row ranges are summed by one workgroup each per 32 x (16 / sizeof(T))
// columns -- 8 row lanes per column group, combined through LDS in lane order -- then one thread per column adds the
// parts in order.
// ---------------------------------------------------------------------------
constexpr int BIAS_PARTS = 64;
size_t bias_grad_partial_bytes(int n) { return n > 0 ? (size_t)BIAS_PARTS * n * sizeof(float) : 0; }

template <typename T>
__global__ __launch_bounds__(256) void bias_grad_partial_kernel(const T* dz, int64_t ld, int rows, int n, float* partial) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[8][32 * V];
  const int cg = threadIdx.x & 31, rl = threadIdx.x >> 5;
  const int col = (blockIdx.x * 32 + cg) * V;
  const int per = (rows + BIAS_PARTS - 1) / BIAS_PARTS;
  const int r0 = blockIdx.y * per, r1 = min(rows, r0 + per);
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  if (col < n)
    for (int r = r0 + rl; r < r1; r += 8) {
      Vec<T> v = ldv(dz + (int64_t)r * ld + col);
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += to_f32(v.v[e]);
    }
#pragma unroll
  for (int e = 0; e < V; ++e) red[rl][cg * V + e] = acc[e];
  __syncthreads();
  if (rl == 0 && col < n) {
#pragma unroll
    for (int e = 0; e < V; ++e) {
      float s = red[0][cg * V + e];
#pragma unroll
      for (int k = 1; k < 8; ++k) s += red[k][cg * V + e];
      partial[(int64_t)blockIdx.y * n + col + e] = s;
    }
  }
}

__global__ __launch_bounds__(256) void bias_grad_finalize_kernel(const float* partial, int n, float* dbias) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= n) return;
  float s = partial[col];
  for (int p = 1; p < BIAS_PARTS; ++p) s += partial[(int64_t)p * n + col];
  dbias[col] += s;
}

hipError_t bias_grad(DType dt, const void* dz, int64_t ld, int rows, int n, float* partial, float* dbias, hipStream_t s) {
  const int V = dt == DT_F32 ? 4 : 8;
  if (rows < 1 || n < 1 || n % V || ld % V || !dz || !partial || !dbias || ((uintptr_t)dz & 15)) return hipErrorInvalidValue;
  const dim3 grid((n / V + 31) / 32, BIAS_PARTS);
  if (dt == DT_F32) hipLaunchKernelGGL((bias_grad_partial_kernel<float>), grid, dim3(256), 0, s, (const float*)dz, ld, rows, n, partial);
  else hipLaunchKernelGGL((bias_grad_partial_kernel<bf16>), grid, dim3(256), 0, s, (const bf16*)dz, ld, rows, n, partial);
  hipLaunchKernelGGL(bias_grad_finalize_kernel, dim3((n + 255) / 256), dim3(256), 0, s, partial, n, dbias);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// activations
// ---------------------------------------------------------------------------
__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.f + erff(u * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_df(float u) {
  return 0.5f * (1.f + erff(u * 0.70710678118654752f)) + u * 0.39894228040143268f * __expf(-0.5f * u * u);
}
__device__ __forceinline__ float sigmoid_f(float g) { return 1.f / (1.f + __expf(-g)); }

// GELU: a = gelu(z).  SwiGLU: a = silu(z[:, :f]) * z[:, f:]
template <typename T, int KIND>
__global__ __launch_bounds__(256) void act_fwd_kernel(ActArgs a) {
  constexpr int V = Vec<T>::N;
  const int fv = a.f / V;
  const int64_t total = (int64_t)a.rows * fv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / fv; const int c = (int)(i % fv) * V;
    Vec<T> o;
    if (KIND == 0) {
      Vec<T> u = ldv((const T*)a.z + r * a.f + c);
#pragma unroll
      for (int e = 0; e < V; ++e) o.v[e] = from_f32<T>(gelu_f(to_f32(u.v[e])));
    } else {
      Vec<T> g = ldv((const T*)a.z + r * 2 * a.f + c), u = ldv((const T*)a.z + r * 2 * a.f + a.f + c);
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const float gv = to_f32(g.v[e]);
        o.v[e] = from_f32<T>(gv * sigmoid_f(gv) * to_f32(u.v[e]));
      }
    }
    stv((T*)a.a + r * a.f + c, o);
  }
}

// GELU: z := da * gelu'(z).  SwiGLU: z[:, :f] := da*u*(sg + g*sg*(1-sg)),  z[:, f:] := da*g*sg
template <typename T, int KIND>
__global__ __launch_bounds__(256) void act_bwd_kernel(ActArgs a) {
  constexpr int V = Vec<T>::N;
  const int fv = a.f / V;
  const int64_t total = (int64_t)a.rows * fv;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / fv; const int c = (int)(i % fv) * V;
    Vec<T> da = ldv((const T*)a.da + r * a.f + c);
    if (KIND == 0) {
      T* zp = (T*)a.z + r * a.f + c;
      Vec<T> u = ldv(zp), o;
#pragma unroll
      for (int e = 0; e < V; ++e) o.v[e] = from_f32<T>(to_f32(da.v[e]) * gelu_df(to_f32(u.v[e])));
      stv(zp, o);
    } else {
      T* gp = (T*)a.z + r * 2 * a.f + c; T* up = gp + a.f;
      Vec<T> g = ldv(gp), u = ldv(up), og, ou;
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const float gv = to_f32(g.v[e]), uv = to_f32(u.v[e]), d = to_f32(da.v[e]);
        const float sg = sigmoid_f(gv);
        og.v[e] = from_f32<T>(d * uv * (sg + gv * sg * (1.f - sg)));
        ou.v[e] = from_f32<T>(d * gv * sg);
      }
      stv(gp, og); stv(up, ou);
    }
  }
}

template <typename T>
static hipError_t act_t(const ActArgs& a, bool bwd, hipStream_t s) {
  constexpr int V = 16 / sizeof(T);
  if (a.f % V != 0 || a.rows <= 0) return hipErrorInvalidValue;
  const int64_t total = (int64_t)a.rows * (a.f / V);
  const int grid = (int)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
  if (!bwd) {
    if (a.kind == 0) hipLaunchKernelGGL((act_fwd_kernel<T, 0>), dim3(grid), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((act_fwd_kernel<T, 1>), dim3(grid), dim3(256), 0, s, a);
  } else {
    if (a.kind == 0) hipLaunchKernelGGL((act_bwd_kernel<T, 0>), dim3(grid), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((act_bwd_kernel<T, 1>), dim3(grid), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t act_fwd(DType dt, const ActArgs& a, hipStream_t s) {
  return dt == DT_F32 ? act_t<float>(a, false, s) : act_t<bf16>(a, false, s);
}
hipError_t act_bwd(DType dt, const ActArgs& a, hipStream_t s) {
  return dt == DT_F32 ? act_t<float>(a, true, s) : act_t<bf16>(a, true, s);
}

// ---------------------------------------------------------------------------
// fill / copy (kernels rather than memset/memcpy nodes, so that a caller may
// capture a schedule into a HIP graph)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* p, size_t nvec, float* tail, size_t ntail) {
  const uint4 z = {0, 0, 0, 0};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) p[i] = z;
  if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0.f;
}

hipError_t fill_zero_f32(float* p, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const size_t nvec = n / 4;
  const size_t want = (nvec + 255) / 256;
  const int grid = (int)(want < 1 ? 1 : (want > 16384 ? 16384 : want));
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, s, (uint4*)p, nvec, p + nvec * 4, n - nvec * 4);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* dst, const uint4* src, size_t nvec) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

template <typename T>
__global__ __launch_bounds__(256) void widen_kernel(float* dst, const T* src, size_t nvec) {
  constexpr int V = Vec<T>::N;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) {
    float v[V];
    ld_row<T>(v, src, (int64_t)i * V, false);
    st_row<T>(dst, (int64_t)i * V, v, true);
  }
}

hipError_t widen_to_f32(DType dt, float* dst, const void* src, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const size_t V = dt == DT_F32 ? 4 : 8;
  if (n % V) return hipErrorInvalidValue;
  const size_t nvec = n / V, want = (nvec + 255) / 256;
  const int grid = (int)(want > 16384 ? 16384 : want);
  if (dt == DT_F32) hipLaunchKernelGGL((widen_kernel<float>), dim3(grid), dim3(256), 0, s, dst, (const float*)src, nvec);
  else hipLaunchKernelGGL((widen_kernel<bf16>), dim3(grid), dim3(256), 0, s, dst, (const bf16*)src, nvec);
  return hipGetLastError();
}

hipError_t copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if (bytes % 16) return hipErrorInvalidValue;
  const size_t nvec = bytes / 16;
  const size_t want = (nvec + 255) / 256;
  const int grid = (int)(want > 16384 ? 16384 : want);
  hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, s, (uint4*)dst, (const uint4*)src, nvec);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Rotary position embedding (the paper's layers are Llama-style): consecutive pairs (2p, 2p+1) of every q and k head
// are rotated by pos * theta^(-2p/hd), pos = position in the sequence; the backward pass applies the transpose.
// The angles' cosines and sines come from a table [s][hd/2] of (cos, sin), built once in double precision.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rope_table_kernel(float2* table, int s, int half, double theta) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)s * half) return;
  const int pos = (int)(i / half), p = (int)(i % half);
  const double ang = (double)pos * pow(theta, -(double)p / (double)half);
  table[i] = make_float2((float)cos(ang), (float)sin(ang));
}

// in place on the first nh heads of every row of x [rows, ld]; one 16-byte vector per thread and step
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T* x, int64_t ld, int64_t rows, int s, int nh, int hd, const float2* table,
                                                   int inverse) {
  constexpr int V = Vec<T>::N;
  const int per_row = nh * hd / V, vec_per_head = hd / V;
  const int64_t total = rows * per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / per_row;
    const int c = (int)(i % per_row);
    const int pos = (int)(row % s), p0 = (c % vec_per_head) * (V / 2);          // first pair index inside the head
    T* ptr = x + row * ld + (int64_t)c * V;
    Vec<T> v = ldv(ptr);
    const float2* t = table + (int64_t)pos * (hd / 2) + p0;
#pragma unroll
    for (int q = 0; q < V / 2; ++q) {
      const float2 cs = t[q];
      const float sn = inverse ? -cs.y : cs.y;
      const float a = to_f32(v.v[2 * q]), b = to_f32(v.v[2 * q + 1]);
      v.v[2 * q] = from_f32<T>(a * cs.x - b * sn);
      v.v[2 * q + 1] = from_f32<T>(a * sn + b * cs.x);
    }
    stv(ptr, v);
  }
}

hipError_t rope_table(float* table, int s, int hd, double theta, hipStream_t st) {
  if (s < 1 || hd < 2 || hd % 2 || !(theta > 0.0) || !table) return hipErrorInvalidValue;
  const int64_t n = (int64_t)s * (hd / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (float2*)table, s, hd / 2, theta);
  return hipGetLastError();
}

hipError_t rope_apply(DType dt, void* x, int64_t ld, int64_t rows, int s, int nh, int hd, const float* table, int inverse,
                      hipStream_t st) {
  const int V = dt == DT_F32 ? 4 : 8;
  if (rows < 1 || s < 1 || nh < 1 || hd % V || ld % V || !x || !table || ((uintptr_t)x & 15)) return hipErrorInvalidValue;
  const int64_t total = rows * (nh * hd / V), want = (total + 255) / 256;
  const int grid = (int)(want > 16384 ? 16384 : want);
  if (dt == DT_F32) hipLaunchKernelGGL((rope_kernel<float>), dim3(grid), dim3(256), 0, st, (float*)x, ld, rows, s, nh, hd, (const float2*)table, inverse);
  else hipLaunchKernelGGL((rope_kernel<bf16>), dim3(grid), dim3(256), 0, st, (bf16*)x, ld, rows, s, nh, hd, (const float2*)table, inverse);
  return hipGetLastError();
}

}  // namespace stg
