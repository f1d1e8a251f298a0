// Fused causal / full attention for gfx950 in bf16 with fp32 softmax: forward
// (online softmax, no s-by-s tensor in HBM) and a deterministic two-kernel
// backward.  K/V (forward, dQ) or Q/dO (dK/dV) tiles are staged through LDS;
// every product runs on v_mfma_f32_32x32x16_bf16.
//
// Orientation trick used throughout: the score block is computed transposed
// (keys x queries in forward / dQ, queries x keys in dK/dV) so that each lane
// owns ONE row of the softmax (forward, dQ) or one key (dK/dV) and the
// probabilities it holds are exactly the 8-wide reduction slices the next MFMA
// wants as an operand -- P and dS never leave registers.  The other operand of
// that MFMA (V^T, K^T, dO^T, Q^T) is fetched from the row-major LDS tile with
// the LDS transpose load ds_read_b64_tr_b16.
//
// Backward is split so that no atomics are needed (bit-reproducible gradients):
//   dQ kernel:    one workgroup per (sequence, head, query tile), loops over key tiles
//   dK/dV kernel: one workgroup per (sequence, kv head, key tile), loops over the query
//                 heads of the group and their query tiles in a fixed order
// both recompute P = exp(S - lse) from the forward's log-sum-exp.
//
// On this chip plain VALU instructions do not overlap with MFMAs of the same wavefront (v_exp_f32 does), and at
// head_dim 128 the softmax arithmetic is ~5 VALU instructions per MFMA, so the kernels keep that arithmetic
// minimal (scale folded into the exponent's fma, first MFMA of a chain takes C = 0 as an inline constant, output
// rescale skipped when no row maximum moved) and dispatch the heaviest causal tiles first.
#include "common.h"

namespace stg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int THREADS = 256;
constexpr int TK = 64;            // rows of one LDS tile (keys in forward / dQ, queries in dK/dV)
constexpr int PADE = 40;          // row padding (elements): 16-byte row reads and transpose reads both spread over banks
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

template <int HD, int NTHR = THREADS> struct Cfg {
  static constexpr int LD = HD + PADE;           // LDS row stride (elements)
  static constexpr int NKK = HD / 16;            // k-steps of a product reducing over head_dim
  static constexpr int NHB = HD / 32;            // 32-wide head_dim blocks of an output
  static constexpr int TILE = TK * LD;           // elements per LDS tile
  static constexpr int CH = TK * HD / 8 / NTHR;    // 16-byte chunks per thread per tile
};

template <int HD, int NTHR> using TileRegs = uint4[Cfg<HD, NTHR>::CH];

// ---- tile movement ----------------------------------------------------------
// rows [row0, row0+TK) of a [*, ld] matrix (HD columns from col0) -> registers; rows >= nrows read as zero
template <int HD, int NTHR = THREADS>
__device__ __forceinline__ void tile_g2r(TileRegs<HD, NTHR>& r, const bf16* __restrict__ base, int64_t ld, int row0,
                                         int nrows, int tid) {
#pragma unroll
  for (int j = 0; j < Cfg<HD, NTHR>::CH; ++j) {
    const int c = tid + NTHR * j;
    const int row = c / (HD / 8), col = (c % (HD / 8)) * 8;
    uint4 v = {0, 0, 0, 0};
    if (row0 + row < nrows) v = *reinterpret_cast<const uint4*>(base + (int64_t)(row0 + row) * ld + col);
    r[j] = v;
  }
}
template <int HD, int NTHR = THREADS>
__device__ __forceinline__ void tile_r2s(const TileRegs<HD, NTHR>& r, bf16* tile, int tid) {
#pragma unroll
  for (int j = 0; j < Cfg<HD, NTHR>::CH; ++j) {
    const int c = tid + NTHR * j;
    *reinterpret_cast<uint4*>(tile + (c / (HD / 8)) * Cfg<HD>::LD + (c % (HD / 8)) * 8) = r[j];
  }
}

// ---- MFMA operand fragments ---------------------------------------------------
// operand with rows = tile rows, reduction over head_dim: lane l -> tile row row0 + l%32, columns kk + (l/32)*8 ..+7
template <int LD>
__device__ __forceinline__ bf16x8 frag_rows(const bf16* tile, int row0, int kk, int lane) {
  return *reinterpret_cast<const bf16x8*>(tile + (row0 + (lane & 31)) * LD + kk + (lane >> 5) * 8);
}
// same operand straight from global memory (kept in registers for the whole kernel); rows >= nrows read as zero
__device__ __forceinline__ bf16x8 frag_rows_global(const bf16* base, int64_t ld, int row0, int nrows, int kk, int lane) {
  const int row = row0 + (lane & 31);
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (bf16)0.f;
  if (row < nrows) z = *reinterpret_cast<const bf16x8*>(base + (int64_t)row * ld + kk + (lane >> 5) * 8);
  return z;
}
// transposed operand: rows = head_dim columns c0 + l%32 of the tile, reduction over tile rows.  The 8 reduction
// slots of lane-half hf = l/32 are tile rows  r0 + 4*hf + {0,1,2,3}  and  r0 + 8 + 4*hf + {0,1,2,3}: the order in
// which a lane holds a 32x32 accumulator block's rows, so a register-resident P / dS block pairs with it directly.
template <int LD>
__device__ __forceinline__ bf16x8 frag_cols_tr(const bf16* tile, int r0, int c0, int lane) {
  const int g = lane >> 4, li = lane & 15;
  const bf16* p = tile + (r0 + (g >> 1) * 4 + (li >> 2)) * LD + c0 + (g & 1) * 16 + (li & 3) * 4;
  typedef s16x4 __attribute__((address_space(3))) * lds_p;
  union { struct { s16x4 a, b; } s; bf16x8 v; } u;
  u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
  u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 8 * LD));
  return u.v;
}

__device__ __forceinline__ bf16x8 pack8(const float* v) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16)v[e];
  return r;
}
__device__ __forceinline__ float xhalf(float v) { return __shfl_xor(v, 32, 64); }
__device__ __forceinline__ void zero(f32x16& a) {
#pragma unroll
  for (int e = 0; e < 16; ++e) a[e] = 0.f;
}
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)
// first product of an accumulation chain: C = 0 as an inline constant, so no registers are cleared beforehand
__device__ __forceinline__ f32x16 mfma0(bf16x8 a, bf16x8 b) {
  const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, z, 0, 0, 0);
}

// row index inside a 32-row accumulator block held in register e by a lane of half hf
__device__ __forceinline__ int acc_row(int e, int hf) { return (e >> 2) * 8 + hf * 4 + (e & 3); }

// ---------------------------------------------------------------------------
// forward: one workgroup = 8 wavefronts x 32 queries of one (sequence, head).  Two wavefronts share a SIMD, so
// one can run its softmax (VALU, exp) while the other runs MFMAs.
// ---------------------------------------------------------------------------
constexpr int FWD_THREADS = 512;
constexpr int FWD_BQ = (FWD_THREADS / 64) * 32;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32; -inf -> 0

template <int HD>
__global__ __launch_bounds__(FWD_THREADS) void attn_fwd_kernel(AttnArgs a) {
  using C = Cfg<HD, FWD_THREADS>;
  __shared__ __attribute__((aligned(16))) bf16 sK[C::TILE];
  __shared__ __attribute__((aligned(16))) bf16 sV[C::TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5;
  constexpr int BQ = FWD_BQ;
  const int nqt = (a.s + BQ - 1) / BQ;
  const int qt = nqt - 1 - blockIdx.y;              // slow grid index: heaviest (latest) query tiles are dispatched first
  const int j = blockIdx.x, ib = blockIdx.z;
  const int d = a.h * HD, dkv = a.hkv * HD, g = j / (a.h / a.hkv);
  const bf16* base = (const bf16*)a.qkv + (int64_t)ib * a.s * a.ld;
  const bf16* qp = base + j * HD;
  const bf16* kp = base + d + g * HD;
  const bf16* vp = base + d + dkv + g * HD;
  const int q0b = qt * BQ, q0w = q0b + wave * 32;
  const int q = q0w + (lane & 31);
  const float sl2 = rsqrtf((float)HD) * LOG2E;

  bf16x8 qf[C::NKK];
#pragma unroll
  for (int kk = 0; kk < C::NKK; ++kk) qf[kk] = frag_rows_global(qp, a.ld, q0w, a.s, kk * 16, lane);

  f32x16 o[C::NHB];
#pragma unroll
  for (int hb = 0; hb < C::NHB; ++hb) zero(o[hb]);
  float m = -1e30f, l = 0.f;                       // running max (in log2 units, scaled) and sum of the lane's query

  const int last_q = min(q0b + BQ, a.s) - 1;
  const int ntiles = a.causal ? last_q / TK + 1 : (a.s + TK - 1) / TK;
  uint4 rk[C::CH], rv[C::CH];
  tile_g2r<HD, FWD_THREADS>(rk, kp, a.ld, 0, a.s, tid);
  tile_g2r<HD, FWD_THREADS>(rv, vp, a.ld, 0, a.s, tid);
  tile_r2s<HD, FWD_THREADS>(rk, sK, tid);
  tile_r2s<HD, FWD_THREADS>(rv, sV, tid);
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const int kv0 = t * TK;
    if (t + 1 < ntiles) {
      tile_g2r<HD, FWD_THREADS>(rk, kp, a.ld, kv0 + TK, a.s, tid);
      tile_g2r<HD, FWD_THREADS>(rv, vp, a.ld, kv0 + TK, a.s, tid);
    }
    const bool active = !a.causal || kv0 <= min(q0w + 32, a.s) - 1;
    if (active && q0w < a.s) {
      // S^T[key][query] for two 32-key blocks
      f32x16 sacc[2];
      sacc[0] = mfma0(frag_rows<C::LD>(sK, 0, 0, lane), qf[0]);
      sacc[1] = mfma0(frag_rows<C::LD>(sK, 32, 0, lane), qf[0]);
#pragma unroll
      for (int kk = 1; kk < C::NKK; ++kk) {
        sacc[0] = MFMA(frag_rows<C::LD>(sK, 0, kk * 16, lane), qf[kk], sacc[0]);
        sacc[1] = MFMA(frag_rows<C::LD>(sK, 32, kk * 16, lane), qf[kk], sacc[1]);
      }
      const bool need_mask = (a.causal && kv0 + TK - 1 > q0w) || kv0 + TK > a.s;
      float p[2][16];
      float mx = -INFINITY;
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float x = sacc[c][e];                       // raw score; sl2 > 0, so the max can be taken before scaling
          if (need_mask) {
            const int key = kv0 + c * 32 + acc_row(e, hf);
            if (key >= a.s || (a.causal && key > q)) x = -INFINITY;
          }
          p[c][e] = x;
          mx = fmaxf(mx, x);
        }
      mx = fmaxf(mx, xhalf(mx));
      const float mn = fmaxf(m, mx * sl2);
      float sum = 0.f;
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) { p[c][e] = fast_exp2(fmaf(p[c][e], sl2, -mn)); sum += p[c][e]; }
      sum += xhalf(sum);
      if (__any(mn != m)) {                          // the running max moved for some query of the wavefront
        const float alpha = fast_exp2(m - mn);
        l *= alpha;
#pragma unroll
        for (int hb = 0; hb < C::NHB; ++hb)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[hb][e] *= alpha;
      }
      l += sum;
      m = mn;
      bf16x8 pf[2][2];
#pragma unroll
      for (int c = 0; c < 2; ++c) { pf[c][0] = pack8(&p[c][0]); pf[c][1] = pack8(&p[c][8]); }
      // O^T[hd][query] += V^T . P^T
#pragma unroll
      for (int hb = 0; hb < C::NHB; ++hb)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
            o[hb] = MFMA(frag_cols_tr<C::LD>(sV, c * 32 + t2 * 16, hb * 32, lane), pf[c][t2], o[hb]);
    }
    __syncthreads();
    if (t + 1 < ntiles) {
      tile_r2s<HD, FWD_THREADS>(rk, sK, tid);
      tile_r2s<HD, FWD_THREADS>(rv, sV, tid);
    }
    __syncthreads();
  }

  if (q < a.s) {
    const float inv = 1.f / l;
    bf16* orow = (bf16*)a.o + ((int64_t)ib * a.s + q) * d + j * HD;
#pragma unroll
    for (int hb = 0; hb < C::NHB; ++hb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[hb][q4 * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + hb * 32 + q4 * 8 + hf * 4) = v;
      }
    if (hf == 0) a.lse[((int64_t)ib * a.h + j) * a.s + q] = (m + log2f(l)) * LN2;
  }
}

// ---------------------------------------------------------------------------
// delta[b,h,i] = sum_t dout[i,h,t] * o[i,h,t]; HD/8 lanes per (row, head)
// ---------------------------------------------------------------------------
template <int HD>
__global__ __launch_bounds__(256) void attn_delta_kernel(AttnArgs a) {
  constexpr int LPR = HD / 8;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t item = gid / LPR;                      // (row, head)
  const int part = (int)(gid % LPR);
  const int64_t nitems = (int64_t)a.b * a.s * a.h;
  float acc = 0.f;
  if (item < nitems) {
    const int64_t row = item / a.h; const int j = (int)(item % a.h);
    const int64_t off = row * a.h * HD + (int64_t)j * HD + part * 8;
    bf16x8 x = *reinterpret_cast<const bf16x8*>((const bf16*)a.dout + off);
    bf16x8 y = *reinterpret_cast<const bf16x8*>((const bf16*)a.o + off);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)x[e] * (float)y[e];
  }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (item < nitems && part == 0) {
    const int64_t row = item / a.h; const int j = (int)(item % a.h);
    const int64_t ib = row / a.s, i = row % a.s;
    a.delta[(ib * a.h + j) * a.s + i] = acc;
  }
}

// ---------------------------------------------------------------------------
// dQ: one workgroup = 8 wavefronts x 32 queries of one (sequence, head); two wavefronts per SIMD so that one
// wavefront's exp / dS arithmetic overlaps the other's MFMAs
// ---------------------------------------------------------------------------
template <int HD>
__global__ __launch_bounds__(FWD_THREADS) void attn_dq_kernel(AttnArgs a) {
  using C = Cfg<HD, FWD_THREADS>;
  __shared__ __attribute__((aligned(16))) bf16 sK[C::TILE];
  __shared__ __attribute__((aligned(16))) bf16 sV[C::TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5;
  constexpr int BQ = FWD_BQ;
  const int nqt = (a.s + BQ - 1) / BQ;
  const int qt = nqt - 1 - blockIdx.y;              // slow grid index: heaviest query tiles first
  const int j = blockIdx.x, ib = blockIdx.z;
  const int d = a.h * HD, dkv = a.hkv * HD, g = j / (a.h / a.hkv);
  const bf16* base = (const bf16*)a.qkv + (int64_t)ib * a.s * a.ld;
  const bf16* qp = base + j * HD;
  const bf16* kp = base + d + g * HD;
  const bf16* vp = base + d + dkv + g * HD;
  const bf16* dop = (const bf16*)a.dout + (int64_t)ib * a.s * d + j * HD;
  const int q0b = qt * BQ, q0w = q0b + wave * 32;
  const float scale = rsqrtf((float)HD), sl2 = scale * LOG2E;
  const int q = q0w + (lane & 31);

  bf16x8 qf[C::NKK], dof[C::NKK];
#pragma unroll
  for (int kk = 0; kk < C::NKK; ++kk) {
    qf[kk] = frag_rows_global(qp, a.ld, q0w, a.s, kk * 16, lane);
    dof[kk] = frag_rows_global(dop, d, q0w, a.s, kk * 16, lane);
  }
  float lse2 = 1e30f, dl = 0.f;                       // rows past the end: P = 0
  if (q < a.s) {
    lse2 = a.lse[((int64_t)ib * a.h + j) * a.s + q] * LOG2E;
    dl = a.delta[((int64_t)ib * a.h + j) * a.s + q];
  }
  f32x16 dq[C::NHB];
#pragma unroll
  for (int hb = 0; hb < C::NHB; ++hb) zero(dq[hb]);

  const int last_q = min(q0b + BQ, a.s) - 1;
  const int ntiles = a.causal ? last_q / TK + 1 : (a.s + TK - 1) / TK;
  uint4 rk[C::CH], rv[C::CH];
  tile_g2r<HD, FWD_THREADS>(rk, kp, a.ld, 0, a.s, tid);
  tile_g2r<HD, FWD_THREADS>(rv, vp, a.ld, 0, a.s, tid);
  tile_r2s<HD, FWD_THREADS>(rk, sK, tid);
  tile_r2s<HD, FWD_THREADS>(rv, sV, tid);
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const int kv0 = t * TK;
    if (t + 1 < ntiles) {
      tile_g2r<HD, FWD_THREADS>(rk, kp, a.ld, kv0 + TK, a.s, tid);
      tile_g2r<HD, FWD_THREADS>(rv, vp, a.ld, kv0 + TK, a.s, tid);
    }
    const bool active = !a.causal || kv0 <= min(q0w + 32, a.s) - 1;
    if (active && q0w < a.s) {
      const bool need_mask = (a.causal && kv0 + TK - 1 > q0w) || kv0 + TK > a.s;
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        if (a.causal && kv0 + c * 32 > q0w + 31) continue;          // the whole 32-key block is in the future
        f32x16 sacc = mfma0(frag_rows<C::LD>(sK, c * 32, 0, lane), qf[0]);             // S^T  = K . Q^T
        f32x16 pacc = mfma0(frag_rows<C::LD>(sV, c * 32, 0, lane), dof[0]);            // dP^T = V . dO^T
#pragma unroll
        for (int kk = 1; kk < C::NKK; ++kk) {
          sacc = MFMA(frag_rows<C::LD>(sK, c * 32, kk * 16, lane), qf[kk], sacc);
          pacc = MFMA(frag_rows<C::LD>(sV, c * 32, kk * 16, lane), dof[kk], pacc);
        }
        float ds[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float p = fast_exp2(sacc[e] * sl2 - lse2);
          if (need_mask) {
            const int key = kv0 + c * 32 + acc_row(e, hf);
            if (key >= a.s || (a.causal && key > q)) p = 0.f;
          }
          ds[e] = p * (pacc[e] - dl);
        }
        const bf16x8 ds0 = pack8(&ds[0]), ds1 = pack8(&ds[8]);
        // dQ^T[hd][query] += K^T . dS^T
#pragma unroll
        for (int hb = 0; hb < C::NHB; ++hb) {
          dq[hb] = MFMA(frag_cols_tr<C::LD>(sK, c * 32, hb * 32, lane), ds0, dq[hb]);
          dq[hb] = MFMA(frag_cols_tr<C::LD>(sK, c * 32 + 16, hb * 32, lane), ds1, dq[hb]);
        }
      }
    }
    __syncthreads();
    if (t + 1 < ntiles) {
      tile_r2s<HD, FWD_THREADS>(rk, sK, tid);
      tile_r2s<HD, FWD_THREADS>(rv, sV, tid);
    }
    __syncthreads();
  }

  if (q < a.s) {
    bf16* row = (bf16*)a.dqkv + ((int64_t)ib * a.s + q) * a.ld + j * HD;
#pragma unroll
    for (int hb = 0; hb < C::NHB; ++hb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[hb][q4 * 4 + e] * scale);
        *reinterpret_cast<bf16x4*>(row + hb * 32 + q4 * 8 + hf * 4) = v;
      }
  }
}

// ---------------------------------------------------------------------------
// dK/dV: one workgroup = NTHR/64 wavefronts x 32 keys of one (sequence, kv head)
// ---------------------------------------------------------------------------
template <int HD, int NTHR>
__global__ __launch_bounds__(NTHR) void attn_dkv_kernel(AttnArgs a) {
  using C = Cfg<HD, NTHR>;
  __shared__ __attribute__((aligned(16))) bf16 sQ[C::TILE];
  __shared__ __attribute__((aligned(16))) bf16 sO[C::TILE];
  __shared__ __attribute__((aligned(16))) float sL[TK];     // lse * log2(e) per query of the tile
  __shared__ __attribute__((aligned(16))) float sD[TK];     // delta per query of the tile
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5;
  constexpr int BKEY = (NTHR / 64) * 32;
  const int kt = blockIdx.y;                              // slow grid index: early key tiles see the most queries, first
  const int g = blockIdx.x, ib = blockIdx.z;
  const int d = a.h * HD, dkv = a.hkv * HD, grp = a.h / a.hkv;
  const bf16* base = (const bf16*)a.qkv + (int64_t)ib * a.s * a.ld;
  const bf16* kp = base + d + g * HD;
  const bf16* vp = base + d + dkv + g * HD;
  const int k0b = kt * BKEY, k0w = k0b + wave * 32;
  const int key = k0w + (lane & 31);
  const float scale = rsqrtf((float)HD), sl2 = scale * LOG2E;

  bf16x8 kf[C::NKK], vf[C::NKK];
#pragma unroll
  for (int kk = 0; kk < C::NKK; ++kk) {
    kf[kk] = frag_rows_global(kp, a.ld, k0w, a.s, kk * 16, lane);
    vf[kk] = frag_rows_global(vp, a.ld, k0w, a.s, kk * 16, lane);
  }
  f32x16 dk[C::NHB], dv[C::NHB];
#pragma unroll
  for (int hb = 0; hb < C::NHB; ++hb) { zero(dk[hb]); zero(dv[hb]); }

  const int t_first = a.causal ? k0b / TK : 0;
  const int nqt = (a.s + TK - 1) / TK;
  const int per_head = nqt - t_first;
  const int niter = per_head * grp;
  uint4 rq[C::CH], ro[C::CH];
  float rl = 0.f, rd = 0.f;

  auto fetch = [&](int it) {
    const int jj = it / per_head, t = t_first + it % per_head;
    const int j = g * grp + jj;
    tile_g2r<HD, NTHR>(rq, base + j * HD, a.ld, t * TK, a.s, tid);
    tile_g2r<HD, NTHR>(ro, (const bf16*)a.dout + (int64_t)ib * a.s * d + j * HD, d, t * TK, a.s, tid);
    if (tid < TK) {
      const int qi = t * TK + tid;
      rl = 1e30f; rd = 0.f;
      if (qi < a.s) {
        rl = a.lse[((int64_t)ib * a.h + j) * a.s + qi] * LOG2E;
        rd = a.delta[((int64_t)ib * a.h + j) * a.s + qi];
      }
    }
  };
  auto stash = [&]() {
    tile_r2s<HD, NTHR>(rq, sQ, tid);
    tile_r2s<HD, NTHR>(ro, sO, tid);
    if (tid < TK) { sL[tid] = rl; sD[tid] = rd; }
  };

  if (niter > 0) { fetch(0); stash(); }
  __syncthreads();

  for (int it = 0; it < niter; ++it) {
    const int t = t_first + it % per_head;
    const int q0 = t * TK;
    if (it + 1 < niter) fetch(it + 1);
    if (k0w < a.s) {
#pragma unroll
      for (int qc = 0; qc < 2; ++qc) {
        if (a.causal && q0 + qc * 32 + 31 < k0w) continue;          // every query of the block precedes every key
        f32x16 sacc = mfma0(frag_rows<C::LD>(sQ, qc * 32, 0, lane), kf[0]);            // S  = Q . K^T
        f32x16 pacc = mfma0(frag_rows<C::LD>(sO, qc * 32, 0, lane), vf[0]);            // dP = dO . V^T
#pragma unroll
        for (int kk = 1; kk < C::NKK; ++kk) {
          sacc = MFMA(frag_rows<C::LD>(sQ, qc * 32, kk * 16, lane), kf[kk], sacc);
          pacc = MFMA(frag_rows<C::LD>(sO, qc * 32, kk * 16, lane), vf[kk], pacc);
        }
        const bool need_mask = a.causal && q0 + qc * 32 < k0w + 31;
        float p[16], ds[16];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(&sL[qc * 32 + e4 * 8 + hf * 4]);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(&sD[qc * 32 + e4 * 8 + hf * 4]);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            float pv = fast_exp2(sacc[e4 * 4 + e] * sl2 - l4[e]);
            if (need_mask && q0 + qc * 32 + e4 * 8 + hf * 4 + e < key) pv = 0.f;
            p[e4 * 4 + e] = pv;
            ds[e4 * 4 + e] = pv * (pacc[e4 * 4 + e] - d4[e]);
          }
        }
        const bf16x8 pf0 = pack8(&p[0]), pf1 = pack8(&p[8]), df0 = pack8(&ds[0]), df1 = pack8(&ds[8]);
#pragma unroll
        for (int hb = 0; hb < C::NHB; ++hb) {
          dv[hb] = MFMA(frag_cols_tr<C::LD>(sO, qc * 32, hb * 32, lane), pf0, dv[hb]);        // dV^T += dO^T . P
          dv[hb] = MFMA(frag_cols_tr<C::LD>(sO, qc * 32 + 16, hb * 32, lane), pf1, dv[hb]);
          dk[hb] = MFMA(frag_cols_tr<C::LD>(sQ, qc * 32, hb * 32, lane), df0, dk[hb]);        // dK^T += Q^T . dS
          dk[hb] = MFMA(frag_cols_tr<C::LD>(sQ, qc * 32 + 16, hb * 32, lane), df1, dk[hb]);
        }
      }
    }
    __syncthreads();
    if (it + 1 < niter) stash();
    __syncthreads();
  }

  if (key < a.s) {
    bf16* row = (bf16*)a.dqkv + ((int64_t)ib * a.s + key) * a.ld + d + g * HD;
#pragma unroll
    for (int hb = 0; hb < C::NHB; ++hb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 vk, vv;
#pragma unroll
        for (int e = 0; e < 4; ++e) { vk[e] = (bf16)(dk[hb][q4 * 4 + e] * scale); vv[e] = (bf16)dv[hb][q4 * 4 + e]; }
        *reinterpret_cast<bf16x4*>(row + hb * 32 + q4 * 8 + hf * 4) = vk;
        *reinterpret_cast<bf16x4*>(row + dkv + hb * 32 + q4 * 8 + hf * 4) = vv;
      }
  }
}

template <int HD>
hipError_t fwd_t(const AttnArgs& a, hipStream_t s) {
  const int nqt = (a.s + FWD_BQ - 1) / FWD_BQ;
  hipLaunchKernelGGL((attn_fwd_kernel<HD>), dim3(a.h, nqt, a.b), dim3(FWD_THREADS), 0, s, a);
  return hipGetLastError();
}

template <int HD>
hipError_t bwd_t(const AttnArgs& a, hipStream_t s) {
  const int64_t lanes = (int64_t)a.b * a.s * a.h * (HD / 8);
  hipLaunchKernelGGL((attn_delta_kernel<HD>), dim3((unsigned)((lanes + 255) / 256)), dim3(256), 0, s, a);
  hipLaunchKernelGGL((attn_dq_kernel<HD>), dim3(a.h, (a.s + FWD_BQ - 1) / FWD_BQ, a.b), dim3(FWD_THREADS), 0, s, a);
    // 256 keys per workgroup (8 wavefronts, two per SIMD) when that still gives two workgroups per CU, else 128
  if ((int64_t)a.b * a.hkv * ((a.s + 255) / 256) >= 512)
    hipLaunchKernelGGL((attn_dkv_kernel<HD, 512>), dim3(a.hkv, (a.s + 255) / 256, a.b), dim3(512), 0, s, a);
  else
    hipLaunchKernelGGL((attn_dkv_kernel<HD, 256>), dim3(a.hkv, (a.s + 127) / 128, a.b), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) {
  if (a.hd != 64 && a.hd != 128) return false;
  if (a.ld % 8 || ((uintptr_t)a.qkv & 15) || ((uintptr_t)a.o & 15)) return false;
  if (a.dout && (((uintptr_t)a.dout & 15) || ((uintptr_t)a.dqkv & 15))) return false;
  return a.b > 0 && a.s > 0 && a.h > 0 && a.hkv > 0 && a.h % a.hkv == 0;
}

hipError_t attn_fwd_mfma(const AttnArgs& a, hipStream_t s) { return a.hd == 128 ? fwd_t<128>(a, s) : fwd_t<64>(a, s); }
hipError_t attn_bwd_mfma(const AttnArgs& a, hipStream_t s) { return a.hd == 128 ? bwd_t<128>(a, s) : bwd_t<64>(a, s); }

}  // namespace stg
