// bf16 MFMA GEMM for gfx950, the three operand layouts of a linear layer's
// forward, input-gradient and weight-gradient products (paper Appendix B):
//
//   NN  C[M,N]  = A[M,K] . B[K,N] (+ R)        forward,  A.W
//   NT  C[M,N]  = A[M,K] . B[N,K]^T            dgrad,    dZ.W^T
//   TN  C[M,N] += A[K,M]^T . B[K,N]   (fp32)   wgrad,    A^T.dZ
//
// Design: 256x256x64 macro tile per workgroup, 8 wavefronts (2x4, two per SIMD),
// each owning a 128x64 sub-tile as 4x2 v_mfma_f32_32x32x16_bf16 accumulators
// (128 fp32 registers per lane).  Global -> register -> LDS through buffer loads
// (hardware range check, no branches) with the next-but-one K tile in flight,
// two LDS buffers and one barrier per K tile; fragments are double-buffered in
// registers and the loop body is an explicit 4-stage software pipeline.  An operand whose
// reduction index is contiguous in memory sits in LDS as [row][k] (padded to
// 72 elements: conflict-free 16-byte fragment reads); an operand whose
// reduction index is the slow one sits as [k][row] (padded to 288) and is read
// with ds_read_b64_tr_b16, the LDS transpose load, so no layout needs a
// transposing copy.  The MFMA is issued with the operands swapped (computes the
// transposed 32x32 block), which leaves every lane with 4 consecutive columns
// of one row: 8-byte bf16 / 16-byte fp32 epilogue accesses.  Workgroup ids are
// remapped so that each XCD (own L2) works on a compact band of tiles.
#include "common.h"

namespace stg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

#ifndef GEMM_EXPERIMENT
#define GEMM_EXPERIMENT 0
#endif

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int KPAD = BK + 8;      // [row][k] layout: 144-byte rows
constexpr int MPAD = BM + 32;     // [k][row] layout: 576-byte rows
constexpr int TILE_ELEMS = BM * KPAD;                      // == BK * MPAD == 18432
static_assert(BM * KPAD == BK * MPAD, "both layouts use the same LDS footprint");
constexpr int TILE_CHUNKS = BM * BK / 8;                   // 16-byte chunks of one operand tile = 2048
constexpr size_t LDS_BYTES = (size_t)4 * TILE_ELEMS * sizeof(bf16);   // A,B x 2 buffers = 147456

enum Epi { EPI_STORE = 0, EPI_RESID = 1, EPI_ACC32 = 2 };

typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned OOB = 0x80000000u;   // any offset >= num_records makes a buffer load return zeros

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// Per-thread byte offsets of its CHUNKS 16-byte pieces of one operand tile at k = 0.  Rows past the end of
// the matrix fall outside the buffer's range by themselves (offset >= rows*ld*2); a piece whose contiguous
// coordinate is out of range is redirected to OOB.  KC: reduction index contiguous in memory.
template <bool KC, int NTHR>
__device__ __forceinline__ void tile_offsets(unsigned (&off)[TILE_CHUNKS / NTHR], int64_t ld, int row0, int rows, int tid) {
#pragma unroll
  for (int j = 0; j < TILE_CHUNKS / NTHR; ++j) {
    const int c = tid + NTHR * j;
    if (KC) {
      const int row = row0 + (c >> 3), k = (c & 7) * 8;
      off[j] = (unsigned)(((int64_t)row * ld + k) * 2);
      if (row >= rows) off[j] = OOB;
    } else {
      const int k = c >> 5, row = row0 + (c & 31) * 8;
      off[j] = row < rows ? (unsigned)(((int64_t)k * ld + row) * 2) : OOB;
    }
  }
}

// one operand tile at reduction offset k0 (a multiple of BK; K % BK == 0 for a KC operand): global -> registers,
// no branches.  OOB + anything below 2 GiB stays out of range; reduction rows >= K of a non-KC operand are past
// the end of the buffer.
template <bool KC, int NCH>
__device__ __forceinline__ void g2r(uint4 (&r)[NCH], __amdgpu_buffer_rsrc_t rsrc, const unsigned (&off)[NCH],
                                    int64_t ld, int k0) {
  const unsigned step = KC ? (unsigned)k0 * 2u : (unsigned)((int64_t)k0 * ld * 2);
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(off[j] + step), 0, 0);
    r[j] = uint4{(unsigned)v[0], (unsigned)v[1], (unsigned)v[2], (unsigned)v[3]};
  }
}

template <bool KC, int NTHR>
__device__ __forceinline__ void r2s(const uint4 (&r)[TILE_CHUNKS / NTHR], bf16* tile, int tid) {
#pragma unroll
  for (int j = 0; j < TILE_CHUNKS / NTHR; ++j) {
    const int c = tid + NTHR * j;
    int off;
    if (KC) off = (c >> 3) * KPAD + (c & 7) * 8; else off = (c >> 5) * MPAD + (c & 31) * 8;
    *reinterpret_cast<uint4*>(tile + off) = r[j];
  }
}

// 32(row) x 16(k) MFMA operand fragment: lane l holds row l%32, k = (l/32)*8 .. +7
template <bool KC>
__device__ __forceinline__ bf16x8 frag(const bf16* tile, int row0, int kk, int lane) {
  if (KC) {
    const bf16* p = tile + (row0 + (lane & 31)) * KPAD + kk + (lane >> 5) * 8;
    return *reinterpret_cast<const bf16x8*>(p);
  } else {
    // transpose load: in a 16-lane group, lane i addresses row (i/4) of a 4(k) x 16(row) block at
    // column 4*(i%4) and receives column i of the block, i.e. 4 consecutive k for its own row
    const int g = lane >> 4, li = lane & 15;
    const bf16* p = tile + (kk + (g >> 1) * 8 + (li >> 2)) * MPAD + row0 + (g & 1) * 16 + (li & 3) * 4;
    typedef s16x4 __attribute__((address_space(3))) * lds_p;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 4 * MPAD));
    union { struct { s16x4 a, b; } s; bf16x8 v; } u;
    u.s.a = lo; u.s.b = hi;
    return u.v;
  }
}

// TN = 32-column accumulator blocks per wavefront: 4 -> 4 wavefronts of 128x128 (one per SIMD, 256 accumulator
// registers), 2 -> 8 wavefronts of 128x64 (two per SIMD, 128 accumulator registers each)
template <bool AKC, bool BKC, int EPI, int TN>
__global__ __launch_bounds__(1024 / TN) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  constexpr int THREADS = 1024 / TN, CHUNKS = TILE_CHUNKS / THREADS, WGN = 8 / TN;   // wave grid 2 x WGN
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave / WGN) * 128, wn = (wave % WGN) * (TN * 32);

  // XCD-aware tile order: consecutive workgroup ids go to different XCDs, so give XCD x the
  // x-th contiguous band of the tile sequence; inside it walk groups of 8 tile rows column by column.
  int bid = blockIdx.x;
  const int nb = tiles_m * tiles_n;
  {
    const int per = nb >> 3, main = per << 3;
    if (bid < main) bid = (bid & 7) * per + (bid >> 3);
  }
  constexpr int GROUP = 8;
  const int in_group = GROUP * tiles_n;
  const int gid = bid / in_group;
  const int first_m = gid * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int tile_m = first_m + (bid % in_group) % gsz;
  const int tile_n = (bid % in_group) / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const bf16* A = (const bf16*)g.A;
  const bf16* B = (const bf16*)g.B;

  // Accumulators start at zero, or -- weight gradients, C += A^T.B -- at the current value of C: the read half of
  // the read-modify-write then travels together with the first operand tiles instead of stalling the epilogue.
  f32x16 acc[4][TN];
  if (EPI == EPI_ACC32) {
    const __amdgpu_buffer_rsrc_t rsC = make_rsrc(g.C, (unsigned)(((int64_t)(g.M - 1) * g.ldc + g.N) * 4));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + wm + i * 32 + (lane & 31);
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + wn + j * 32 + q * 8 + (lane >> 5) * 4;
          const unsigned off = (m < g.M && n < g.N) ? (unsigned)(((int64_t)m * g.ldc + n) * 4) : OOB;
          const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsC, (int)off, 0, 0));
          acc[i][j][q * 4] = v[0]; acc[i][j][q * 4 + 1] = v[1]; acc[i][j][q * 4 + 2] = v[2]; acc[i][j][q * 4 + 3] = v[3];
        }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  }

  // buffer descriptors cover exactly the rows that exist: KC operand = [rows, ld], other = [K, ld]
  const __amdgpu_buffer_rsrc_t rsA = make_rsrc(A, (unsigned)(((int64_t)((AKC ? g.M : g.K) - 1) * g.lda + (AKC ? g.K : g.M)) * 2));
  const __amdgpu_buffer_rsrc_t rsB = make_rsrc(B, (unsigned)(((int64_t)((BKC ? g.N : g.K) - 1) * g.ldb + (BKC ? g.K : g.N)) * 2));
  unsigned offa[CHUNKS], offb[CHUNKS];
  tile_offsets<AKC, THREADS>(offa, g.lda, m0, g.M, tid);
  tile_offsets<BKC, THREADS>(offb, g.ldb, n0, g.N, tid);

  uint4 ra[CHUNKS], rb[CHUNKS];
  const int nk = (g.K + BK - 1) / BK;
  g2r<AKC, CHUNKS>(ra, rsA, offa, g.lda, 0);
  g2r<BKC, CHUNKS>(rb, rsB, offb, g.ldb, 0);
  r2s<AKC, THREADS>(ra, smem, tid);
  r2s<BKC, THREADS>(rb, smem + TILE_ELEMS, tid);
  g2r<AKC, CHUNKS>(ra, rsA, offa, g.lda, BK);
  g2r<BKC, CHUNKS>(rb, rsB, offb, g.ldb, BK);
  __syncthreads();

  // Software pipeline, one K tile (4 k-steps of 16) per trip, fragments double-buffered in registers:
  //   S0  read frags k1 | MFMA k0            S2  read frags k3 | write tile t+1 to the other LDS buffer | MFMA k2
  //   S1  read frags k2 | MFMA k1            -- barrier --
  //                                          S3  read frags k0 of tile t+1 | issue global loads of tile t+2 | MFMA k3
  // Loads past the last K tile return zeros (buffer range check), so the loop needs no branches.
  constexpr int NREADS = (AKC ? 4 : 8) + (BKC ? TN : 2 * TN);   // LDS read instructions per k-step
  constexpr int NMFMA = 4 * TN;                                 // MFMAs per k-step
  bf16x8 fa[2][4], fb[2][TN];
#define LOAD_FRAGS(buf, sa_, sb_, kk_)                                              \
  _Pragma("unroll") for (int i = 0; i < 4; ++i) fa[buf][i] = frag<AKC>(sa_, wm + i * 32, kk_, lane); \
  _Pragma("unroll") for (int j = 0; j < TN; ++j) fb[buf][j] = frag<BKC>(sb_, wn + j * 32, kk_, lane);
#define MFMA_STEP(buf)                                                               \
  _Pragma("unroll") for (int i = 0; i < 4; ++i)                                      \
  _Pragma("unroll") for (int j = 0; j < TN; ++j)                                     \
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
  // scheduling hint: `n` instructions of class `mask`, spread evenly over the NMFMA MFMAs of a stage
#define SPREAD(mask, n)                                                                              \
  __builtin_amdgcn_sched_group_barrier(mask, (n) / 4, 0);                                            \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 4, 0);                                         \
  __builtin_amdgcn_sched_group_barrier(mask, (2 * (n)) / 4 - (n) / 4, 0);                            \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 4, 0);                                         \
  __builtin_amdgcn_sched_group_barrier(mask, (3 * (n)) / 4 - (2 * (n)) / 4, 0);                      \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 4, 0);                                         \
  __builtin_amdgcn_sched_group_barrier(mask, (n) - (3 * (n)) / 4, 0);                                \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 4, 0);
  // the same with a second instruction class riding along: n reads and m others per stage
#define SPREAD2(mask2, n, m)                                                                         \
  __builtin_amdgcn_sched_group_barrier(0x100, (n) / 4, 0);                                           \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 8, 0);                                         \
  __builtin_amdgcn_sched_group_barrier(mask2, (m) / 4, 0);                                           \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 4 - NMFMA / 8, 0);                             \
  __builtin_amdgcn_sched_group_barrier(0x100, (2 * (n)) / 4 - (n) / 4, 0);                           \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 8, 0);                                         \
  __builtin_amdgcn_sched_group_barrier(mask2, (m) / 4, 0);                                           \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 4 - NMFMA / 8, 0);                             \
  __builtin_amdgcn_sched_group_barrier(0x100, (3 * (n)) / 4 - (2 * (n)) / 4, 0);                     \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 8, 0);                                         \
  __builtin_amdgcn_sched_group_barrier(mask2, (m) / 4, 0);                                           \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 4 - NMFMA / 8, 0);                             \
  __builtin_amdgcn_sched_group_barrier(0x100, (n) - (3 * (n)) / 4, 0);                               \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 8, 0);                                         \
  __builtin_amdgcn_sched_group_barrier(mask2, (m) / 4, 0);                                           \
  __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 4 - NMFMA / 8, 0);

  LOAD_FRAGS(0, smem, smem + TILE_ELEMS, 0)
  for (int kt = 0; kt < nk; ++kt) {
    const bf16* sa = smem + (kt & 1) * 2 * TILE_ELEMS;
    const bf16* sb = sa + TILE_ELEMS;
    bf16* na = smem + ((kt + 1) & 1) * 2 * TILE_ELEMS;
    bf16* nb = na + TILE_ELEMS;
    // S0
    LOAD_FRAGS(1, sa, sb, 16)
    MFMA_STEP(0)
    SPREAD(0x100, NREADS)
    __builtin_amdgcn_sched_barrier(0);
    // S1
    LOAD_FRAGS(0, sa, sb, 32)
    MFMA_STEP(1)
    SPREAD(0x100, NREADS)
    __builtin_amdgcn_sched_barrier(0);
    // S2: LDS reads first (the compiler will not move a read below a write it cannot prove disjoint)
    LOAD_FRAGS(1, sa, sb, 48)
    r2s<AKC, THREADS>(ra, na, tid);
    r2s<BKC, THREADS>(rb, nb, tid);
    MFMA_STEP(0)
    __builtin_amdgcn_sched_group_barrier(0x100, NREADS / 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 8, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, NREADS - NREADS / 2, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, NMFMA / 8, 0);
    __builtin_amdgcn_sched_group_barrier(0x200, 2 * CHUNKS / 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, (NMFMA - 2 * (NMFMA / 8)) / 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x200, 2 * CHUNKS / 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, (NMFMA - 2 * (NMFMA / 8)) / 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x200, 2 * CHUNKS / 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, (NMFMA - 2 * (NMFMA / 8)) / 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x200, 2 * CHUNKS / 4, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, (NMFMA - 2 * (NMFMA / 8)) / 4, 0);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    // S3
    LOAD_FRAGS(0, na, nb, 0)
#if GEMM_EXPERIMENT == 2      // timing experiment only: keep re-reading K tile 0 (cache resident)
    g2r<AKC, CHUNKS>(ra, rsA, offa, g.lda, 0);
    g2r<BKC, CHUNKS>(rb, rsB, offb, g.ldb, 0);
#else
    g2r<AKC, CHUNKS>(ra, rsA, offa, g.lda, (kt + 2) * BK);
    g2r<BKC, CHUNKS>(rb, rsB, offb, g.ldb, (kt + 2) * BK);
#endif
    MFMA_STEP(1)
    SPREAD2(0x020, NREADS, 2 * CHUNKS)
    __builtin_amdgcn_sched_barrier(0);
  }
#undef LOAD_FRAGS
#undef MFMA_STEP
#undef SPREAD
#undef SPREAD2

  // epilogue: acc[i][j][e] = C[m][n],  m = m0+wm+i*32 + lane%32,  n = n0+wn+j*32 + (e/4)*8 + (lane/32)*4 + e%4
#if GEMM_EXPERIMENT == 3      // timing experiment only: no epilogue stores unless a value is NaN
  if (!(acc[0][0][0] != acc[0][0][0])) return;
#endif
  const int row_l = lane & 31, col_l = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + wm + i * 32 + row_l;
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn + j * 32 + q * 8 + col_l;
        if (n >= g.N) continue;          // N % 8 == 0 and n % 4 == 0: the 4 columns are in or out together
        f32x4 v = {acc[i][j][q * 4], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
        if (EPI == EPI_ACC32) {
          *reinterpret_cast<f32x4*>((float*)g.C + (int64_t)m * g.ldc + n) = v;   // acc already holds C + A^T.B
        } else {
          if (EPI == EPI_RESID && g.R) {
            if (g.r_f32) {
              v += *reinterpret_cast<const f32x4*>((const float*)g.R + (int64_t)m * g.ldr + n);
            } else {
              bf16x4 r = *reinterpret_cast<const bf16x4*>((const bf16*)g.R + (int64_t)m * g.ldr + n);
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] += (float)r[e];
            }
          }
          if (EPI == EPI_RESID && g.c_f32) {
            *reinterpret_cast<f32x4*>((float*)g.C + (int64_t)m * g.ldc + n) = v;
          } else {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
            *reinterpret_cast<bf16x4*>((bf16*)g.C + (int64_t)m * g.ldc + n) = o;
          }
        }
      }
    }
  }
}

// Eight wavefronts of 128x64 measured 3-5 % faster than four of 128x128 on the stage's GEMM shapes: the second
// wavefront per SIMD issues MFMAs while the first waits on LDS or at the barrier.
constexpr int WAVE_COLS = 2;

template <bool AKC, bool BKC, int EPI, int TN>
hipError_t launch_tn(const GemmArgs& g, hipStream_t s) {
  static bool attr_set = false;
  auto kern = gemm_mfma_kernel<AKC, BKC, EPI, TN>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(1024 / TN), LDS_BYTES, s, g, tiles_m, tiles_n);
  return hipGetLastError();
}

template <bool AKC, bool BKC, int EPI>
hipError_t launch(const GemmArgs& g, hipStream_t s) {
  return launch_tn<AKC, BKC, EPI, WAVE_COLS>(g, s);
}

}  // namespace

bool gemm_mfma_supported(const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return false;
  auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  if (!al16(g.A) || !al16(g.B) || !al16(g.C) || (g.R && !al16(g.R))) return false;
  if (g.lda % 8 || g.ldb % 8 || g.ldc % 4 || (g.R && g.ldr % 4) || g.N % 8) return false;
  const int64_t lim = (int64_t)1 << 30;   // operand byte offsets are 32-bit buffer offsets below 2 GiB
  const int64_t a_rows = g.mode == GEMM_TN ? g.K : g.M, b_rows = g.mode == GEMM_NT ? g.N : g.K;
  if (a_rows * g.lda >= lim || b_rows * g.ldb >= lim) return false;
  if (g.acc_f32 && (int64_t)g.M * g.ldc >= lim / 2) return false;   // C is read through a 32-bit byte offset too
  switch (g.mode) {
    case GEMM_NN: return g.K % BK == 0 && !g.acc_f32;
    case GEMM_NT: return g.K % BK == 0 && !g.acc_f32 && !g.R && !g.c_f32;
    case GEMM_TN: return g.M % 8 == 0 && g.acc_f32 && !g.R && !g.c_f32;
  }
  return false;
}

hipError_t gemm_mfma(const GemmArgs& g, hipStream_t s) {
  switch (g.mode) {
    case GEMM_NN: return (g.R || g.c_f32) ? launch<true, false, EPI_RESID>(g, s) : launch<true, false, EPI_STORE>(g, s);
    case GEMM_NT: return launch<true, true, EPI_STORE>(g, s);
    case GEMM_TN: return launch<false, false, EPI_ACC32>(g, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace stg
