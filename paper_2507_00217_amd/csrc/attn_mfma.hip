// Fused causal / full attention for gfx950 in bf16 with fp32 softmax: forward
// (online softmax, no s-by-s tensor in HBM) and a deterministic two-kernel
// backward.  K/V (forward, dQ) or Q/dO (dK/dV) tiles go global -> LDS directly (buffer
// loads with the LDS bit) into two buffers, one barrier per tile; every product
// runs on v_mfma_f32_32x32x16_bf16.
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
//   dQ kernel:    one workgroup per (sequence, head, query tile), loops over key tiles; also forms
//                 delta = rowsum(dO * O) of its queries and leaves it in the scratch for the second kernel
//   dK/dV kernel: one workgroup per (sequence, kv head, key tile), loops over the query
//                 heads of the group and their query tiles in a fixed order
// both recompute P = exp(S - lse) from the forward's log-sum-exp.
//
// Measured on this chip: plain vector instructions do not overlap with MFMAs of the same wavefront (an interleaved
// stream runs slower than the two parts back to back; v_exp_f32 is the exception), but those of another wavefront on
// the same SIMD do, each MFMA costing that other wavefront about nine issue cycles.  So forward and dQ run two
// wavefronts per SIMD, keep the softmax arithmetic minimal (scale folded into the exponent's fma, first MFMA of a
// chain takes C = 0 as an inline constant, output rescale skipped when no row maximum moved, row sums two at a time
// with the bf16 dot instruction, masks as one compare per element against a per-tile bound, absolute LDS addresses
// so that a fragment read is one register plus an immediate) and read LDS fragments a few MFMAs ahead of their use.
// The heaviest causal tiles are dispatched first.
#include "common.h"

#include <utility>

namespace stg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int TK = 64;            // rows of one LDS tile (keys in forward / dQ, queries in dK/dV)
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

typedef __attribute__((address_space(3))) char lds_char;
typedef int rsrc_words __attribute__((ext_vector_type(4)));

// LDS tile: TK rows of HD bf16, unpadded, filled by buffer loads that write LDS directly (lane l of a wavefront
// lands at the wavefront's LDS address + 16*l, out-of-range lanes store zeros).  The 16-byte piece c (8 columns)
// of row r sits in slot r*PPR + (c ^ swz(r)); the swizzle makes both ways of reading the tile conflict-free:
//   rows as MFMA operand rows (16 consecutive rows, same piece): 16 different 16-byte bank groups
//   transpose reads (4 consecutive rows, 64 contiguous bytes each): 4 different 64-byte bank groups
template <int HD> struct Geo {
  static constexpr int PPR = HD / 8;             // 16-byte pieces per row
  static constexpr int ROWB = HD * 2;            // bytes per row
  static constexpr int TILEB = TK * ROWB;        // bytes per tile
  static constexpr int NKK = HD / 16;            // k-steps of a product reducing over head_dim
  static constexpr int NHB = HD / 32;            // 32-wide head_dim blocks of an output
  __device__ static __forceinline__ int swz(int r) {
    return HD == 128 ? (((r & 3) << 2) | ((r >> 2) & 3)) : ((((r >> 1) & 1) << 2) | ((r >> 2) & 3));
  }
};

__device__ __forceinline__ rsrc_words raw_rsrc(const void* base, unsigned bytes) {
  const uint64_t a = (uint64_t)base;
  return rsrc_words{(int)(unsigned)a, (int)(unsigned)((a >> 32) & 0xffffu), (int)bytes, 0x00020000};
}
// Inline assembly on purpose: with the builtin the compiler cannot tell these LDS writes from the fragment reads
// of the other buffer and drains the vector-memory counter before every LDS read.  Completion is awaited by hand
// (vmcnt(0) before the barrier that publishes a tile).  m0 = the wavefront's LDS destination.
__device__ __forceinline__ void load_to_lds_b128(rsrc_words rsrc, unsigned lds_addr, unsigned voffset) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(lds_addr), "v"(voffset), "s"(rsrc) : "memory");
}
__device__ __forceinline__ void load_to_lds_b32(rsrc_words rsrc, unsigned lds_addr, unsigned voffset) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, 0 offen lds" :: "s"(lds_addr), "v"(voffset), "s"(rsrc) : "memory");
}

// Per-thread byte offsets (relative to row 0 of the tile's first row, column 0 of the head) of the pieces it
// fetches: load j of wavefront w fills slots (j*NW + w)*64 .. +63.
template <int HD, int NTHR, int ROWS = TK>
__device__ __forceinline__ void tile_offsets(unsigned (&off)[ROWS * (HD / 8) / NTHR], int64_t ld, int wave, int lane) {
  using G = Geo<HD>;
#pragma unroll
  for (int j = 0; j < ROWS * G::PPR / NTHR; ++j) {
    const int s = (j * (NTHR / 64) + wave) * 64 + lane;
    const int r = s / G::PPR, c = (s % G::PPR) ^ G::swz(r);
    off[j] = (unsigned)(((int64_t)r * ld + c * 8) * 2);
  }
}
// rows [row0, row0+TK) of the matrix behind `rsrc` -> LDS tile; the descriptor ends with the last real row, so rows
// past it are out of range and store zeros.  `wave` must be wave-uniform.
template <int HD, int NTHR, int ROWS = TK>
__device__ __forceinline__ void tile_g2s(lds_char* tile, rsrc_words rsrc, const unsigned (&off)[ROWS * (HD / 8) / NTHR],
                                         int64_t ld, int row0, int wave) {
  const unsigned step = (unsigned)((int64_t)row0 * ld * 2);
#pragma unroll
  for (int j = 0; j < ROWS * (HD / 8) / NTHR; ++j)
    load_to_lds_b128(rsrc, (unsigned)(size_t)(tile + (j * (NTHR / 64) + wave) * 1024), off[j] + step);
}
// descriptor of one head's [nrows, HD] slice of a row-major matrix with row stride ld (elements)
__device__ __forceinline__ rsrc_words head_rsrc(const bf16* p, int64_t ld, int nrows, int hd) {
  return raw_rsrc(p, (unsigned)(((int64_t)(nrows - 1) * ld + hd) * 2));
}

// ---- MFMA operand fragments ---------------------------------------------------
// Per-lane byte offsets inside a tile.
//   rows-type operand (rows = tile rows, reduction over head_dim: lane l -> tile row rb + l%32, columns
//   16*ks + (l/32)*8 ..+7):  ro[ks], plus rb * ROWB for the row block
//   transposed operand (rows = head_dim columns hb*32 + l%32, reduction over 16 tile rows r0..r0+15; the 8 reduction
//   slots of lane-half hf = l/32 are tile rows r0 + 4*hf + {0,1,2,3} and r0 + 8 + 4*hf + {0,1,2,3}: the order in
//   which a lane holds a 32x32 accumulator block's rows, so a register-resident P / dS block pairs with it
//   directly):  co[hb][0 or 1] for the two 4-row groups, plus r0 * ROWB (r0 a multiple of 16)
template <int HD>
struct FragOff {
  unsigned ro[HD / 16];
  unsigned co[HD / 32][2];
  // `lds`: the workgroup's LDS base; the offsets are absolute LDS addresses, so a read's address is one register
  // plus an immediate
  __device__ __forceinline__ void init(int lane, lds_char* lds) {
    using G = Geo<HD>;
    const unsigned base = (unsigned)(size_t)lds;
    const int r = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < G::NKK; ++ks) ro[ks] = base + (unsigned)(r * G::ROWB + (((2 * ks + hf) ^ G::swz(r)) << 4));
    const int g = lane >> 4, li = lane & 15;
#pragma unroll
    for (int hb = 0; hb < G::NHB; ++hb)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int row = (g >> 1) * 4 + (li >> 2) + 8 * u;
        const int piece = hb * 4 + (g & 1) * 2 + ((li & 3) >> 1);
        co[hb][u] = base + (unsigned)(row * G::ROWB + ((piece ^ G::swz(row)) << 4) + (li & 1) * 8);
      }
  }
  __device__ __forceinline__ void hop(int bytes) {
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) ro[ks] += bytes;
#pragma unroll
    for (int hb = 0; hb < HD / 32; ++hb) { co[hb][0] += bytes; co[hb][1] += bytes; }
  }
};
template <int HD>
__device__ __forceinline__ bf16x8 frag_rows(lds_char* lds, const FragOff<HD>& f, int tile_off, int rb, int ks) {
  return *(__attribute__((address_space(3))) const bf16x8*)(size_t)(f.ro[ks] + (unsigned)(tile_off + rb * Geo<HD>::ROWB));
}
template <int HD>
__device__ __forceinline__ bf16x8 frag_cols_tr(lds_char* lds, const FragOff<HD>& f, int tile_off, int r0, int hb) {
  typedef s16x4 __attribute__((address_space(3))) * lds_p;
  union { struct { s16x4 a, b; } s; bf16x8 v; } u;
  u.s.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(size_t)(f.co[hb][0] + (unsigned)(tile_off + r0 * Geo<HD>::ROWB)));
  u.s.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(size_t)(f.co[hb][1] + (unsigned)(tile_off + r0 * Geo<HD>::ROWB)));
  return u.v;
}
// rows-type operand straight from global memory (kept in registers for the whole kernel); rows >= nrows read as zero
__device__ __forceinline__ bf16x8 frag_rows_global(const bf16* base, int64_t ld, int row0, int nrows, int kk, int lane) {
  const int row = row0 + (lane & 31);
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (bf16)0.f;
  if (row < nrows) z = *reinterpret_cast<const bf16x8*>(base + (int64_t)row * ld + kk + (lane >> 5) * 8);
  return z;
}

__device__ __forceinline__ bf16x8 pack8(const float* v) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16)v[e];
  return r;
}
// The value held by the lane 32 further on (or back): v_permlane32_swap exchanges the upper half of one register with
// the lower half of another, one vector instruction instead of a round trip through the LDS crossbar.  Given v twice, the
// first result holds the partner's value in lanes 32-63 and the second in lanes 0-31.  (The second copy is made opaque
// and the two results are only ever selected between, never combined with each other: the compiler folded a sum of the
// two results into twice the first.)
__device__ __forceinline__ float xhalf(float v, int hf) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  unsigned w = u;
  asm volatile("" : "+v"(w));
  const auto r = __builtin_amdgcn_permlane32_swap(u, w, false, false);
  return __builtin_bit_cast(float, hf ? r[0] : r[1]);
}
__device__ __forceinline__ float half_max(float v, int hf) { return fmaxf(v, xhalf(v, hf)); }
__device__ __forceinline__ float half_sum(float v, int hf) { return v + xhalf(v, hf); }
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// acc + sum of the 8 elements of v (v_dot2c_f32_bf16 against (1, 1): exact products, fp32 accumulation)
__device__ __forceinline__ float dot_ones(bf16x8 v, float acc) {
  bf16x2 one;
  one[0] = (bf16)1.f; one[1] = (bf16)1.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    bf16x2 pr;
    pr[0] = v[2 * i]; pr[1] = v[2 * i + 1];
    acc = __builtin_amdgcn_fdot2_f32_bf16(pr, one, acc, false);
  }
  return acc;
}
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
// Forward and dQ come with 8 wavefronts (256 queries) or 4 (128 queries) per workgroup.  Two workgroups of 4 share
// a CU, so either way two wavefronts sit on each SIMD; 8 read every K/V tile once for twice the queries and are faster
// when there is plenty of work, 4 give twice as many workgroups and win when 8 would leave CUs idle.  A third shape
// for grids smaller still: 4 wavefronts on 64 queries, two per 32-query block, each taking one 32-key half of every
// K/V tile (template parameter KS = 2); what the two halves hold is merged through LDS after the last tile.
constexpr int FWD_WIDE = 512, FWD_NARROW = 256;
constexpr int fwd_bq(int nthr, int ks = 1) { return (nthr / 64) * 32 / ks; }

// Which query tile (forward, dQ: the later, the more keys it sees) the workgroup of dispatch rank `rank` takes.
// Plain order is heaviest first.  `fold`: the heavier half first, heaviest first, then the lighter half, lightest
// first -- for grids that are resident all at once with two workgroups per CU, so that a CU's second workgroup is as
// light as its first is heavy (ranks r and r + nh add up to the same work) instead of the chip waiting for the CUs that
// drew two heavy ones.
__device__ __forceinline__ int tile_of_rank(int rank, int n, int fold) {
  const int nh = (n + 1) >> 1;
  return (!fold || rank < nh) ? n - 1 - rank : rank - nh;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32; -inf -> 0

#define SCHED_FENCE __builtin_amdgcn_sched_barrier(0)
// One key tile of the forward for one wavefront (32 queries x 64 keys).  LDS fragment reads run ahead of the MFMAs
// that consume them (K fragments three k-steps ahead; the first V^T fragments are fetched before the softmax
// arithmetic and land while it runs), so a wavefront does not sit out one LDS round trip per MFMA.
template <int HD, int BUF, int NC = 2>
__device__ __forceinline__ void fwd_tile(lds_char* lds, const FragOff<HD>& fo, const bf16x8 (&qf)[HD / 16], f32x16 (&o)[HD / 32],
                                         float& m, float& l, int kv0, int q, int hf, int s, int causal, float sl2, bool need_mask) {
  using G = Geo<HD>;
  constexpr int KT = BUF, VT = BUF + G::TILEB, AHEAD = 3, NPV = G::NHB * 2 * NC, VA = 4;
  // S^T[key][query] for NC 32-key blocks
  bf16x8 kf[AHEAD + 1][NC];
#pragma unroll
  for (int kk = 0; kk < AHEAD; ++kk)
#pragma unroll
    for (int c = 0; c < NC; ++c) kf[kk][c] = frag_rows<HD>(lds, fo, KT, c * 32, kk);
  f32x16 sacc[NC];
#pragma unroll
  for (int kk = 0; kk < G::NKK; ++kk) {
    if (kk + AHEAD < G::NKK) {
#pragma unroll
      for (int c = 0; c < NC; ++c) kf[(kk + AHEAD) % (AHEAD + 1)][c] = frag_rows<HD>(lds, fo, KT, c * 32, kk + AHEAD);
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (kk == 0) sacc[c] = mfma0(kf[0][c], qf[0]);
      else sacc[c] = MFMA(kf[kk % (AHEAD + 1)][c], qf[kk], sacc[c]);
    }
    SCHED_FENCE;
  }
  // step i of the P.V product: head_dim block i % NHB (consecutive MFMAs hit different accumulators), 16-key part i / NHB
  bf16x8 vf[VA];
#pragma unroll
  for (int i = 0; i < VA; ++i) vf[i] = frag_cols_tr<HD>(lds, fo, VT, (i / G::NHB) * 16, i % G::NHB);
  SCHED_FENCE;
  // key kv0 + c*32 + acc_row(e, hf) is masked when it is past the end or (causal) after the lane's query: one bound
  // per tile, compared with compile-time constants; the branch only wraps in-place selects
  if (need_mask) {
    const int bound = min(causal ? q - kv0 : 0x7fffffff, s - 1 - kv0) - hf * 4;
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (c * 32 + acc_row(e, 0) > bound) sacc[c][e] = -INFINITY;
  }
  float mx = -INFINITY;                           // raw scores; sl2 > 0, so the max can be taken before scaling
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[c][e]);
  float p[NC][16];
  mx = half_max(mx, hf);
  const float mn = fmaxf(m, mx * sl2);
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) p[c][e] = fast_exp2(fmaf(sacc[c][e], sl2, -mn));
  if (__any(mn != m)) {                          // the running max moved for some query of the wavefront
    const float alpha = fast_exp2(m - mn);
    l *= alpha;
#pragma unroll
    for (int hb = 0; hb < G::NHB; ++hb)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[hb][e] *= alpha;
  }
  bf16x8 pf[NC][2];
#pragma unroll
  for (int c = 0; c < NC; ++c) { pf[c][0] = pack8(&p[c][0]); pf[c][1] = pack8(&p[c][8]); }
  // row sum of the probabilities as rounded for the P.V product (so the weights applied to V sum to one exactly),
  // two per instruction
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) sum = dot_ones(pf[c][t2], sum);
  sum = half_sum(sum, hf);
  l += sum;
  m = mn;
  SCHED_FENCE;
  // O^T[hd][query] += V^T . P^T
#pragma unroll
  for (int i = 0; i < NPV; ++i) {
    const bf16x8 v = vf[i % VA];
    if (i + VA < NPV) {
      const int n = i + VA;
      vf[i % VA] = frag_cols_tr<HD>(lds, fo, VT, (n / G::NHB) * 16, n % G::NHB);
    }
    o[i % G::NHB] = MFMA(v, pf[(i / G::NHB) >> 1][(i / G::NHB) & 1], o[i % G::NHB]);
    SCHED_FENCE;
  }
}

// KS = 2 (small grids): two wavefronts per 32 queries, each taking one 32-key half of every key tile, so that a
// workgroup of 4 wavefronts covers only 64 queries and there are twice as many workgroups (and still two wavefronts on
// every SIMD); the halves' (O, m, l) are merged through LDS at the end.
template <int HD, int FWD_THREADS, int KS>
__global__ __launch_bounds__(FWD_THREADS, 2) void attn_fwd_kernel(AttnArgs a, int fold) {
  using G = Geo<HD>;
  constexpr int KT = 0, VT = G::TILEB, BUFB = 2 * G::TILEB;   // two buffers of (K tile, V tile)
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char* lds = (lds_char*)smem_raw;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int BQ = fwd_bq(FWD_THREADS, KS), KW = TK / KS;
  const int qb = KS == 2 ? wave >> 1 : wave, kh = KS == 2 ? wave & 1 : 0;   // query block, key half
  const int nqt = (a.s + BQ - 1) / BQ;
  const int qt = tile_of_rank(blockIdx.y / a.b, nqt, fold);   // slow grid index: heavy (late) query tiles are dispatched first
  const int j = blockIdx.x, ib = blockIdx.y % a.b;
  const int d = a.h * HD, dkv = a.hkv * HD, g = j / (a.h / a.hkv);
  const bf16* base = (const bf16*)a.qkv + (int64_t)ib * a.s * a.ld;
  const bf16* qp = base + j * HD;
  const rsrc_words rsK = head_rsrc(base + d + g * HD, a.ld, a.s, HD);
  const rsrc_words rsV = head_rsrc(base + d + dkv + g * HD, a.ld, a.s, HD);
  const int q0b = qt * BQ, q0w = q0b + qb * 32;
  const int q = q0w + (lane & 31);
  const float sl2 = rsqrtf((float)HD) * LOG2E;

  const int last_q = min(q0b + BQ, a.s) - 1;
  const int ntiles = a.causal ? last_q / TK + 1 : (a.s + TK - 1) / TK;
  unsigned off[TK * G::PPR / FWD_THREADS];
  tile_offsets<HD, FWD_THREADS>(off, a.ld, wave, lane);
  tile_g2s<HD, FWD_THREADS>(lds + KT, rsK, off, a.ld, 0, wave);
  tile_g2s<HD, FWD_THREADS>(lds + VT, rsV, off, a.ld, 0, wave);
  if (ntiles > 1) {
    tile_g2s<HD, FWD_THREADS>(lds + BUFB + KT, rsK, off, a.ld, TK, wave);
    tile_g2s<HD, FWD_THREADS>(lds + BUFB + VT, rsV, off, a.ld, TK, wave);
  }

  bf16x8 qf[G::NKK];
#pragma unroll
  for (int kk = 0; kk < G::NKK; ++kk) qf[kk] = frag_rows_global(qp, a.ld, q0w, a.s, kk * 16, lane);

  f32x16 o[G::NHB];
#pragma unroll
  for (int hb = 0; hb < G::NHB; ++hb) zero(o[hb]);
  float m = -1e30f, l = 0.f;                       // running max (in log2 units, scaled) and sum of the lane's query

  FragOff<HD> fo;
  fo.init(lane, lds);
  if (KS == 2) fo.hop(kh * 32 * G::ROWB);           // this wavefront's half of every tile
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  // Per key tile: compute from one buffer while the next tile lands in the other; then wait for it, one barrier
  // (every wavefront is done with this buffer), and refill this buffer with the tile after next.  The loop body
  // covers two tiles so that the buffer is a compile-time part of every LDS address.
  auto step = [&](int t, auto buf) {
    constexpr int BUF = decltype(buf)::value;
    const int kv0 = t * TK, kvw = kv0 + kh * 32;     // first key of the tile, of the wavefront's part of it
    const bool active = kvw < a.s && (!a.causal || kvw <= min(q0w + 32, a.s) - 1);
    if (active && q0w < a.s) {
      const bool need_mask = (a.causal && kvw + KW - 1 > q0w) || kvw + KW > a.s;
      fwd_tile<HD, BUF, 2 / KS>(lds, fo, qf, o, m, l, kvw, q, hf, a.s, a.causal, sl2, need_mask);
    }
    __builtin_amdgcn_s_waitcnt(0);                  // tile t+1 has landed (issued a whole tile ago), own LDS reads done
    __syncthreads();
    if (t + 2 < ntiles) {
      tile_g2s<HD, FWD_THREADS>(lds + BUF + KT, rsK, off, a.ld, kv0 + 2 * TK, wave);
      tile_g2s<HD, FWD_THREADS>(lds + BUF + VT, rsV, off, a.ld, kv0 + 2 * TK, wave);
    }
  };
  for (int t = 0; t < ntiles; t += 2) {
    step(t, std::integral_constant<int, 0>{});
    if (t + 1 < ntiles) step(t + 1, std::integral_constant<int, BUFB>{});
  }

  if constexpr (KS == 2) {
    // The loop's last barrier has passed: nobody reads the tiles any more and no load is in flight.  The second half's
    // wavefront leaves its (O, m, l) in LDS ([piece][lane] of 16 bytes), the first half's folds them into its own.
    constexpr int OB = G::NHB * 4 * 1024;            // bytes of one wavefront's O: NHB * 4 pieces of 16 bytes per lane
    static_assert(2 * (OB + 512) <= 4 * G::TILEB, "the merge area fits the tile buffers");
    lds_char* mo = lds + qb * (OB + 512) + lane * 16;
    lds_char* ml = lds + qb * (OB + 512) + OB + lane * 8;
    if (kh == 1) {
#pragma unroll
      for (int hb = 0; hb < G::NHB; ++hb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          *(__attribute__((address_space(3))) f32x4*)(mo + (hb * 4 + q4) * 1024) =
              f32x4{o[hb][q4 * 4], o[hb][q4 * 4 + 1], o[hb][q4 * 4 + 2], o[hb][q4 * 4 + 3]};
      *(__attribute__((address_space(3))) f32x2*)ml = f32x2{m, l};
    }
    __syncthreads();
    if (kh == 1) return;
    const f32x2 other = *(__attribute__((address_space(3))) const f32x2*)ml;
    const float mn = fmaxf(m, other.x);
    const float a0 = fast_exp2(m - mn), a1 = fast_exp2(other.x - mn);   // a half that saw no key has m = -1e30, l = 0, O = 0
    l = l * a0 + other.y * a1;
#pragma unroll
    for (int hb = 0; hb < G::NHB; ++hb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 v = *(__attribute__((address_space(3))) const f32x4*)(mo + (hb * 4 + q4) * 1024);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[hb][q4 * 4 + e] = o[hb][q4 * 4 + e] * a0 + v[e] * a1;
      }
    m = mn;
  }
  if (q < a.s) {
    const float inv = 1.f / l;
    bf16* orow = (bf16*)a.o + ((int64_t)ib * a.s + q) * d + j * HD;
#pragma unroll
    for (int hb = 0; hb < G::NHB; ++hb)
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

// One 32-key block of the dQ pass for one wavefront (32 queries), fragment reads running ahead of the MFMAs like
// in the forward.
template <int HD, int BUF>
__device__ __forceinline__ void dq_block(lds_char* lds, const FragOff<HD>& fo, const bf16x8 (&qf)[HD / 16], const bf16x8 (&dof)[HD / 16],
                                         f32x16 (&dq)[HD / 32], int c, int kv0, int q, int hf, int s, int causal, float sl2,
                                         float lse2, float dl, bool need_mask) {
  using G = Geo<HD>;
  constexpr int KT = BUF, VT = BUF + G::TILEB, AHEAD = 3, NDQ = G::NHB * 2, VA = 4;
  bf16x8 kf[AHEAD + 1][2];                                          // [ring slot][K rows, V rows]
#pragma unroll
  for (int kk = 0; kk < AHEAD; ++kk) { kf[kk][0] = frag_rows<HD>(lds, fo, KT, c * 32, kk); kf[kk][1] = frag_rows<HD>(lds, fo, VT, c * 32, kk); }
  f32x16 sacc, pacc;
#pragma unroll
  for (int kk = 0; kk < G::NKK; ++kk) {
    if (kk + AHEAD < G::NKK) {
      kf[(kk + AHEAD) % (AHEAD + 1)][0] = frag_rows<HD>(lds, fo, KT, c * 32, kk + AHEAD);
      kf[(kk + AHEAD) % (AHEAD + 1)][1] = frag_rows<HD>(lds, fo, VT, c * 32, kk + AHEAD);
    }
    if (kk == 0) { sacc = mfma0(kf[0][0], qf[0]); pacc = mfma0(kf[0][1], dof[0]); }          // S^T = K . Q^T, dP^T = V . dO^T
    else {
      sacc = MFMA(kf[kk % (AHEAD + 1)][0], qf[kk], sacc);
      pacc = MFMA(kf[kk % (AHEAD + 1)][1], dof[kk], pacc);
    }
    SCHED_FENCE;
  }
  // step i of dQ^T[hd][query] += K^T . dS^T: head_dim block i % NHB, 16-key half i / NHB
  bf16x8 tf[VA];
#pragma unroll
  for (int i = 0; i < VA; ++i) tf[i] = frag_cols_tr<HD>(lds, fo, KT, c * 32 + (i / G::NHB) * 16, i % G::NHB);
  SCHED_FENCE;
  float ds[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) ds[e] = fast_exp2(fmaf(sacc[e], sl2, -lse2));
  if (need_mask) {                                                  // one bound per block against compile-time constants
    const int bound = min(causal ? q - kv0 : 0x7fffffff, s - 1 - kv0) - hf * 4 - c * 32;
#pragma unroll
    for (int e = 0; e < 16; ++e)
      if (acc_row(e, 0) > bound) ds[e] = 0.f;
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) ds[e] *= pacc[e] - dl;
  const bf16x8 dsf[2] = {pack8(&ds[0]), pack8(&ds[8])};
  SCHED_FENCE;
#pragma unroll
  for (int i = 0; i < NDQ; ++i) {
    const bf16x8 v = tf[i % VA];
    if (i + VA < NDQ) {
      const int n = i + VA;
      tf[i % VA] = frag_cols_tr<HD>(lds, fo, KT, c * 32 + (n / G::NHB) * 16, n % G::NHB);
    }
    dq[i % G::NHB] = MFMA(v, dsf[i / G::NHB], dq[i % G::NHB]);
    SCHED_FENCE;
  }
}

// ---------------------------------------------------------------------------
// dQ: one workgroup = 8 wavefronts x 32 queries of one (sequence, head); two wavefronts per SIMD so that one
// wavefront's exp / dS arithmetic overlaps the other's MFMAs
// ---------------------------------------------------------------------------
template <int HD, int FWD_THREADS, int KS>
__global__ __launch_bounds__(FWD_THREADS, 2) void attn_dq_kernel(AttnArgs a, int fold) {
  using G = Geo<HD>;
  constexpr int KT = 0, VT = G::TILEB, BUFB = 2 * G::TILEB;   // two buffers of (K tile, V tile)
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char* lds = (lds_char*)smem_raw;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int BQ = fwd_bq(FWD_THREADS, KS);
  const int qb = KS == 2 ? wave >> 1 : wave, kh = KS == 2 ? wave & 1 : 0;   // query block, key half (as in the forward)
  const int nqt = (a.s + BQ - 1) / BQ;
  const int qt = tile_of_rank(blockIdx.y / a.b, nqt, fold);   // slow grid index: heavy query tiles first
  const int j = blockIdx.x, ib = blockIdx.y % a.b;
  const int d = a.h * HD, dkv = a.hkv * HD, g = j / (a.h / a.hkv);
  const bf16* base = (const bf16*)a.qkv + (int64_t)ib * a.s * a.ld;
  const bf16* qp = base + j * HD;
  const rsrc_words rsK = head_rsrc(base + d + g * HD, a.ld, a.s, HD);
  const rsrc_words rsV = head_rsrc(base + d + dkv + g * HD, a.ld, a.s, HD);
  const bf16* dop = (const bf16*)a.dout + (int64_t)ib * a.s * d + j * HD;
  const int q0b = qt * BQ, q0w = q0b + qb * 32;
  const float scale = rsqrtf((float)HD), sl2 = scale * LOG2E;
  const int q = q0w + (lane & 31);

  const int last_q = min(q0b + BQ, a.s) - 1;
  const int ntiles = a.causal ? last_q / TK + 1 : (a.s + TK - 1) / TK;
  unsigned off[TK * G::PPR / FWD_THREADS];
  tile_offsets<HD, FWD_THREADS>(off, a.ld, wave, lane);
  tile_g2s<HD, FWD_THREADS>(lds + KT, rsK, off, a.ld, 0, wave);
  tile_g2s<HD, FWD_THREADS>(lds + VT, rsV, off, a.ld, 0, wave);
  if (ntiles > 1) {
    tile_g2s<HD, FWD_THREADS>(lds + BUFB + KT, rsK, off, a.ld, TK, wave);
    tile_g2s<HD, FWD_THREADS>(lds + BUFB + VT, rsV, off, a.ld, TK, wave);
  }

  bf16x8 qf[G::NKK], dof[G::NKK];
#pragma unroll
  for (int kk = 0; kk < G::NKK; ++kk) {
    qf[kk] = frag_rows_global(qp, a.ld, q0w, a.s, kk * 16, lane);
    dof[kk] = frag_rows_global(dop, d, q0w, a.s, kk * 16, lane);
  }
  // delta = rowsum(dO * O) of the lane's query, formed here from the dO fragments already in registers: a lane holds 8
  // of every 16 columns of its row, the lane 32 further on the other 8.  Written out for the dK/dV kernel.
  float lse2 = 1e30f, dl = 0.f;                       // rows past the end: P = 0
  {
    const bf16* op = (const bf16*)a.o + (int64_t)ib * a.s * d + j * HD;
    float part = 0.f;
#pragma unroll
    for (int kk = 0; kk < G::NKK; ++kk) {
      const bf16x8 of = frag_rows_global(op, d, q0w, a.s, kk * 16, lane);
#pragma unroll
      for (int e = 0; e < 8; ++e) part = fmaf((float)dof[kk][e], (float)of[e], part);
    }
    dl = half_sum(part, hf);
  }
  if (q < a.s) {
    lse2 = a.lse[((int64_t)ib * a.h + j) * a.s + q] * LOG2E;
    if (hf == 0 && kh == 0) a.delta[((int64_t)ib * a.h + j) * a.s + q] = dl;
  }
  f32x16 dq[G::NHB];
#pragma unroll
  for (int hb = 0; hb < G::NHB; ++hb) zero(dq[hb]);

  FragOff<HD> fo;
  fo.init(lane, lds);
  if (KS == 2) fo.hop(kh * 32 * G::ROWB);           // this wavefront's half of every tile
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  // two tiles per loop body, so that the buffer is a compile-time part of every LDS address
  auto step = [&](int t, auto buf) {
    constexpr int BUF = decltype(buf)::value;
    const int kv0 = t * TK;
    const int kvw = kv0 + kh * 32;                    // first key of the wavefront's part of the tile
    const bool active = kvw < a.s && (!a.causal || kvw <= min(q0w + 32, a.s) - 1);
    if (active && q0w < a.s) {
      if constexpr (KS == 2) {
        const bool need_mask = (a.causal && kvw + 31 > q0w) || kvw + 32 > a.s;
        dq_block<HD, BUF>(lds, fo, qf, dof, dq, 0, kvw, q, hf, a.s, a.causal, sl2, lse2, dl, need_mask);
      } else {
        const bool need_mask = (a.causal && kv0 + TK - 1 > q0w) || kv0 + TK > a.s;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          if (a.causal && kv0 + c * 32 > q0w + 31) continue;          // the whole 32-key block is in the future
          dq_block<HD, BUF>(lds, fo, qf, dof, dq, c, kv0, q, hf, a.s, a.causal, sl2, lse2, dl, need_mask);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (t + 2 < ntiles) {
      tile_g2s<HD, FWD_THREADS>(lds + BUF + KT, rsK, off, a.ld, kv0 + 2 * TK, wave);
      tile_g2s<HD, FWD_THREADS>(lds + BUF + VT, rsV, off, a.ld, kv0 + 2 * TK, wave);
    }
  };
  for (int t = 0; t < ntiles; t += 2) {
    step(t, std::integral_constant<int, 0>{});
    if (t + 1 < ntiles) step(t + 1, std::integral_constant<int, BUFB>{});
  }

  if constexpr (KS == 2) {      // add the second key half's dQ to the first's, through LDS (the tiles are no longer read)
    static_assert(2 * G::NHB * 4 * 1024 <= 4 * G::TILEB, "the merge area fits the tile buffers");
    lds_char* mo = lds + qb * (G::NHB * 4 * 1024) + lane * 16;
    if (kh == 1) {
#pragma unroll
      for (int hb = 0; hb < G::NHB; ++hb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          *(__attribute__((address_space(3))) f32x4*)(mo + (hb * 4 + q4) * 1024) =
              f32x4{dq[hb][q4 * 4], dq[hb][q4 * 4 + 1], dq[hb][q4 * 4 + 2], dq[hb][q4 * 4 + 3]};
    }
    __syncthreads();
    if (kh == 1) return;
#pragma unroll
    for (int hb = 0; hb < G::NHB; ++hb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 v = *(__attribute__((address_space(3))) const f32x4*)(mo + (hb * 4 + q4) * 1024);
#pragma unroll
        for (int e = 0; e < 4; ++e) dq[hb][q4 * 4 + e] += v[e];
      }
  }
  if (q < a.s) {
    bf16* row = (bf16*)a.dqkv + ((int64_t)ib * a.s + q) * a.ld + j * HD;
#pragma unroll
    for (int hb = 0; hb < G::NHB; ++hb)
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
// dK/dV: one workgroup = 128 keys of one (sequence, kv head) = 4 key blocks of 32, each worked on by TWO wavefronts
// that share a SIMD (wavefronts w and w+4):
//   the dV wavefront:  S = Q.K^T, P = exp(S - lse),                       dV^T += dO^T.P      16 MFMAs per 32 queries
//   the dK wavefront:  dP = dO.V^T, dS = P (dP - delta),                  dK^T += Q^T.dS      16 MFMAs per 32 queries
// P is computed once: the dV wavefront leaves each 32 x 32 block of it (fp32, its own accumulator layout, which is the dK
// wavefront's too) in a 4 KiB LDS slot of the pair and the dK wavefront picks it up -- a one-slot queue between two
// wavefronts of the same workgroup, a produced and a consumed count in LDS (written right behind the block's writes or
// reads: the LDS executes a wavefront's instructions in order); the waits are bounded spins on those counts (the
// producer never waits for anything but the slot to be free, so they end).  What the split buys: each role fits the
// 256-register budget of two wavefronts per SIMD with every accumulator in ordinary registers, and the vector
// arithmetic of one role runs under the MFMAs of the other -- a single wavefront cannot overlap the two.
// The workgroup walks the query heads of its group and their 128-query tiles (Q, dO, lse, delta of a tile go global ->
// LDS directly, two buffers, one barrier per tile).
// ---------------------------------------------------------------------------
// TQ = keys per workgroup = queries per tile: 128 (8 wavefronts, one workgroup per CU) or, for small grids, 64
// (4 wavefronts, two workgroups per CU: twice as many workgroups for the same number of resident wavefronts)
constexpr int DKV_TQ = 128, DKV_TQ_SMALL = 64;
// early key tiles see the most queries: plain order is kt = rank; folded (see tile_of_rank) the heavy half first, then
// the light half, lightest first
__device__ __forceinline__ int key_tile_of_rank(int rank, int n, int fold) { return n - 1 - tile_of_rank(rank, n, fold); }

// acc = sum over head_dim of rows(tile `TILE`, rows rb..rb+31) x bfr (the wavefront's K or V fragments); fragment
// reads run three k-steps ahead
template <int HD, int TILE>
__device__ __forceinline__ void dkv_rows_product(lds_char* lds, const FragOff<HD>& fo, int rb, const bf16x8 (&bfr)[HD / 16], f32x16& acc) {
  using G = Geo<HD>;
  constexpr int AHEAD = 3;
  bf16x8 f[AHEAD + 1];
#pragma unroll
  for (int kk = 0; kk < AHEAD; ++kk) f[kk] = frag_rows<HD>(lds, fo, TILE, rb, kk);
#pragma unroll
  for (int kk = 0; kk < G::NKK; ++kk) {
    if (kk + AHEAD < G::NKK) f[(kk + AHEAD) % (AHEAD + 1)] = frag_rows<HD>(lds, fo, TILE, rb, kk + AHEAD);
    if (kk == 0) acc = mfma0(f[0], bfr[0]);
    else acc = MFMA(f[kk % (AHEAD + 1)], bfr[kk], acc);
    SCHED_FENCE;
  }
}
// the same for two products at once (S from the Q tile, dP from the dO tile), their MFMAs alternating
template <int HD, int TILE_A, int TILE_B>
__device__ __forceinline__ void dkv_rows_product2(lds_char* lds, const FragOff<HD>& fo, int rb, const bf16x8 (&bfa)[HD / 16],
                                                  const bf16x8 (&bfb)[HD / 16], f32x16& acca, f32x16& accb) {
  using G = Geo<HD>;
  constexpr int AHEAD = 3;
  bf16x8 f[AHEAD + 1][2];
#pragma unroll
  for (int kk = 0; kk < AHEAD; ++kk) { f[kk][0] = frag_rows<HD>(lds, fo, TILE_A, rb, kk); f[kk][1] = frag_rows<HD>(lds, fo, TILE_B, rb, kk); }
#pragma unroll
  for (int kk = 0; kk < G::NKK; ++kk) {
    if (kk + AHEAD < G::NKK) {
      f[(kk + AHEAD) % (AHEAD + 1)][0] = frag_rows<HD>(lds, fo, TILE_A, rb, kk + AHEAD);
      f[(kk + AHEAD) % (AHEAD + 1)][1] = frag_rows<HD>(lds, fo, TILE_B, rb, kk + AHEAD);
    }
    if (kk == 0) { acca = mfma0(f[0][0], bfa[0]); accb = mfma0(f[0][1], bfb[0]); }
    else { acca = MFMA(f[kk % (AHEAD + 1)][0], bfa[kk], acca); accb = MFMA(f[kk % (AHEAD + 1)][1], bfb[kk], accb); }
    SCHED_FENCE;
  }
}
// out[hb]^T += (tile `TILE`, rows rb..rb+31)^T . w, w = the 32 x 32 block of P or dS held as two bf16 fragments;
// the first transposed fragments must already be in tf[] (read before the vector arithmetic that made w)
template <int HD, int TILE>
__device__ __forceinline__ void dkv_tr_read(lds_char* lds, const FragOff<HD>& fo, int rb, bf16x8 (&tf)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) tf[i] = frag_cols_tr<HD>(lds, fo, TILE, rb + (i / Geo<HD>::NHB) * 16, i % Geo<HD>::NHB);
}
template <int HD, int TILE>
__device__ __forceinline__ void dkv_tr_product(lds_char* lds, const FragOff<HD>& fo, int rb, bf16x8 (&tf)[4], const bf16x8 (&w)[2],
                                               f32x16 (&out)[HD / 32]) {
  using G = Geo<HD>;
  constexpr int N = G::NHB * 2, VA = 4;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const bf16x8 v = tf[i % VA];
    if (i + VA < N) {
      const int n = i + VA;
      tf[i % VA] = frag_cols_tr<HD>(lds, fo, TILE, rb + (n / G::NHB) * 16, n % G::NHB);
    }
    out[i % G::NHB] = MFMA(v, w[i / G::NHB], out[i % G::NHB]);
    SCHED_FENCE;
  }
}

template <int HD, int TQ>
__global__ __launch_bounds__(TQ * 4, 2) void attn_dkv_kernel(AttnArgs a, int nsplit, int fold) {
  using G = Geo<HD>;
  constexpr int NTHR = TQ * 4, NB = TQ / 32, NKW = TQ / 32, TILEB = TQ * G::ROWB;   // NKW key blocks, two wavefronts each
  // two buffers of (Q tile, dO tile, lse of the tile's queries, delta of the tile's queries)
  constexpr int QT = 0, OT = TILEB, LT = 2 * TILEB, DT = LT + TQ * 4, BUFB = DT + TQ * 4;
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  lds_char* lds = (lds_char*)smem_raw;
  const int tid = threadIdx.x, lane = tid & 63, hf = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int role = wave / NKW, kw = wave % NKW;          // role 0: dV and the producer of P (on the older wavefront), role 1: dK; with 8 wavefronts kw and kw+4 share a SIMD
  const int nkt = (a.s + TQ - 1) / TQ;
  const int kt = key_tile_of_rank(blockIdx.y / a.b, nkt, fold);   // slow grid index: heavy (early) key tiles first
  // grid.x = KV heads x splits: this workgroup takes `grp` of the query heads of KV head g, starting at head j0
  const int g = blockIdx.x / nsplit, sp = blockIdx.x % nsplit, ib = blockIdx.y % a.b;
  const int d = a.h * HD, dkv = a.hkv * HD, grp = a.h / a.hkv / nsplit, j0 = g * (a.h / a.hkv) + sp * grp;
  const bf16* base = (const bf16*)a.qkv + (int64_t)ib * a.s * a.ld;
  const bf16* dobase = (const bf16*)a.dout + (int64_t)ib * a.s * d;
  const bf16* kp = base + d + g * HD;
  const bf16* vp = base + d + dkv + g * HD;
  const int k0b = kt * TQ, k0w = k0b + kw * 32;
  const int key = k0w + (lane & 31);
  const float scale = rsqrtf((float)HD), sl2 = scale * LOG2E;

  const int t_first = a.causal ? kt : 0;              // keys per workgroup = queries per tile: the diagonal query tile has the key tile's index
  const int per_head = nkt - t_first;
  const int niter = per_head * grp;
  // Per-thread offsets of the pieces it fetches: load j covers rows j*SWEEP + (its wavefront's and lane's row inside
  // a sweep); SWEEP is a multiple of 16, so the swizzle -- and with it the column -- is the same for every j and
  // one offset per matrix is enough.
  constexpr int NLD = TQ * G::PPR / NTHR, SWEEP = NTHR / G::PPR;
  static_assert(SWEEP % 16 == 0, "swizzle period");
  unsigned offq0, offo0;
  {
    const int sl = wave * 64 + lane, r = sl / G::PPR, c = (sl % G::PPR) ^ G::swz(r);
    offq0 = (unsigned)(((int64_t)r * a.ld + c * 8) * 2);
    offo0 = (unsigned)(((int64_t)r * d + c * 8) * 2);
  }
  auto tile_fetch = [&](lds_char* tile, rsrc_words rsrc, unsigned off0, int64_t ld, int row0) {
#pragma unroll
    for (int j = 0; j < NLD; ++j)
      load_to_lds_b128(rsrc, (unsigned)(size_t)(tile + (j * (NTHR / 64) + wave) * 1024),
                       off0 + (unsigned)((int64_t)(row0 + j * SWEEP) * ld * 2));
  };
  // iteration `it` = (query head jj of the group, query tile t): its Q and dO tiles, lse and delta -> buffer at `buf`
  auto fetch = [&](int it, lds_char* buf) {
    const int jj = it / per_head, t = t_first + it % per_head;
    const int j = j0 + jj;
    tile_fetch(buf + QT, head_rsrc(base + j * HD, a.ld, a.s, HD), offq0, a.ld, t * TQ);
    tile_fetch(buf + OT, head_rsrc(dobase + j * HD, d, a.s, HD), offo0, d, t * TQ);
    if (wave < TQ / 64) {   // 64 floats per load; queries past the end read as zero, and so do their Q and dO rows
      const int64_t row = ((int64_t)ib * a.h + j) * a.s;
      const unsigned vo = (unsigned)((t * TQ + wave * 64 + lane) * 4);
      load_to_lds_b32(raw_rsrc(a.lse + row, (unsigned)a.s * 4u), (unsigned)(size_t)(buf + LT + wave * 256), vo);
      load_to_lds_b32(raw_rsrc(a.delta + row, (unsigned)a.s * 4u), (unsigned)(size_t)(buf + DT + wave * 256), vo);
    }
  };
  if (niter > 0) fetch(0, lds);
  if (niter > 1) fetch(1, lds + BUFB);

  FragOff<HD> fo;
  fo.init(lane, lds);
  lds_char* cur = lds;                                // buffer being read, refilled after the barrier (wave-uniform)
  lds_char* ldp = lds + LT + hf * 16;                 // this lane's lse values of the current buffer; delta follows TQ*4 later
  int hopb = BUFB;
  typedef __attribute__((address_space(3))) const f32x4* lds_f4;
  // the pair's P slot ([e4][lane] f32x4) and its counts: produced = blocks written, consumed = blocks read
  lds_char* pslot = lds + 2 * BUFB + kw * 4096 + lane * 16;
  volatile __attribute__((address_space(3))) int* produced = (volatile __attribute__((address_space(3))) int*)(lds + 2 * BUFB + NKW * 4096) + kw;
  volatile __attribute__((address_space(3))) int* consumed = produced + NKW;
  if (tid < 2 * NKW) ((volatile __attribute__((address_space(3))) int*)(lds + 2 * BUFB + NKW * 4096))[tid] = 0;   // published by the barrier below
  auto wait_for = [&](volatile __attribute__((address_space(3))) int* count, int value) {
    for (int guard = 0; *count != value && guard < (1 << 20); ++guard) __builtin_amdgcn_s_sleep(1);
    asm volatile("" ::: "memory");                       // nothing of what follows is read or written ahead of the wait
  };
  int nblk = 0;                                          // 32 x 32 blocks of P handled so far

  // end of an iteration: the next tiles have landed and every wavefront is done with this buffer; refill it
  auto turn = [&](int it) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (it + 2 < niter) fetch(it + 2, cur);
    fo.hop(hopb);
    cur += hopb;
    ldp += hopb;
    hopb = -hopb;
  };
  // P of elements e4*4 .. +3 of query block qc (element e is query q0 + qc*32 + e4*8 + hf*4 + e).  Only the diagonal
  // tile needs the causal mask: an element is masked when its query is before the lane's key, i.e. e < lim.
  // (l4: the lse values of those queries, read from LDS ahead of the product that makes sacc -- read where they are
  // used, each of the four loads would cost the wavefront a full LDS round trip)
  auto probs4 = [&](const f32x16& sacc, const f32x4& l4, int qc, int e4, bool diag, int lim0, float (&pv)[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) pv[e] = fast_exp2(fmaf(sacc[e4 * 4 + e], sl2, -LOG2E * l4[e]));
    if (diag) {
      asm volatile("" ::: "memory");                  // keep this a (wave-uniform) branch: it is rarely taken
      const int lim = lim0 - qc * 32 - e4 * 8;
#pragma unroll
      for (int e = 0; e < 4; ++e) pv[e] = e < lim ? 0.f : pv[e];
    }
  };

  bf16x8 kf[G::NKK];
#pragma unroll
  for (int kk = 0; kk < G::NKK; ++kk) kf[kk] = frag_rows_global(kp, a.ld, k0w, a.s, kk * 16, lane);
  f32x16 acc[G::NHB];                                  // dV^T or dK^T of the wavefront's 32 keys
#pragma unroll
  for (int hb = 0; hb < G::NHB; ++hb) zero(acc[hb]);

  if (role == 0) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int it = 0; it < niter; ++it) {
      const int q0 = (t_first + it % per_head) * TQ;
      const bool diag = a.causal && it % per_head == 0;          // wave-uniform
      const int lim0 = key - q0 - hf * 4;
#pragma unroll
      for (int qc = 0; qc < NB; ++qc) {
        f32x4 l4[4];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) l4[e4] = *reinterpret_cast<lds_f4>(ldp + (qc * 32 + e4 * 8) * 4);
        f32x16 sacc;
        dkv_rows_product<HD, QT>(lds, fo, qc * 32, kf, sacc);
        bf16x8 tf[4];
        dkv_tr_read<HD, OT>(lds, fo, qc * 32, tf);
        SCHED_FENCE;
        float p[16];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
          float pv[4];
          probs4(sacc, l4[e4], qc, e4, diag, lim0, pv);
#pragma unroll
          for (int e = 0; e < 4; ++e) p[e4 * 4 + e] = pv[e];
        }
        wait_for(consumed, nblk);                      // the slot is free
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4)
          *(__attribute__((address_space(3))) f32x4*)(pslot + e4 * 1024) = f32x4{p[e4 * 4], p[e4 * 4 + 1], p[e4 * 4 + 2], p[e4 * 4 + 3]};
        asm volatile("" ::: "memory");                 // the LDS executes a wavefront's instructions in order: the count
        *produced = ++nblk;                            // is written after the block, no wait in between
        asm volatile("" ::: "memory");
        const bf16x8 pf[2] = {pack8(&p[0]), pack8(&p[8])};
        SCHED_FENCE;
        dkv_tr_product<HD, OT>(lds, fo, qc * 32, tf, pf, acc);          // dV^T += dO^T . P
      }
      turn(it);
    }
  } else {
    bf16x8 vf[G::NKK];
#pragma unroll
    for (int kk = 0; kk < G::NKK; ++kk) vf[kk] = frag_rows_global(vp, a.ld, k0w, a.s, kk * 16, lane);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int it = 0; it < niter; ++it) {
#pragma unroll
      for (int qc = 0; qc < NB; ++qc) {
        f32x4 d4[4];                                    // delta of the block's queries, ahead of the product (see probs4)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) d4[e4] = *reinterpret_cast<lds_f4>(ldp + (DT - LT) + (qc * 32 + e4 * 8) * 4);
        f32x16 pacc;
        dkv_rows_product<HD, OT>(lds, fo, qc * 32, vf, pacc);                     // dP = dO.V^T
        bf16x8 tf[4];
        dkv_tr_read<HD, QT>(lds, fo, qc * 32, tf);
        SCHED_FENCE;
        wait_for(produced, nblk + 1);                  // the partner has left this block's P (masked where causal) in the slot
        f32x4 pv[4];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) pv[e4] = *(__attribute__((address_space(3))) const f32x4*)(pslot + e4 * 1024);
        asm volatile("" ::: "memory");                 // in-order LDS: the slot has been read by the time the count is
        *consumed = ++nblk;                            // written, whenever the data reaches the registers
        asm volatile("" ::: "memory");
        float ds[16];
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
#pragma unroll
          for (int e = 0; e < 4; ++e) ds[e4 * 4 + e] = pv[e4][e] * (pacc[e4 * 4 + e] - d4[e4][e]);
        }
        const bf16x8 df[2] = {pack8(&ds[0]), pack8(&ds[8])};
        SCHED_FENCE;
        dkv_tr_product<HD, QT>(lds, fo, qc * 32, tf, df, acc);          // dK^T += Q^T . dS
      }
      turn(it);
    }
  }

  // role 0 holds dV, role 1 holds dK (still to be scaled)
  if (key < a.s) {
    const float osc = role ? scale : 1.f;
    if (nsplit == 1) {
      bf16* row = (bf16*)a.dqkv + ((int64_t)ib * a.s + key) * a.ld + d + g * HD + (role ? 0 : dkv);
#pragma unroll
      for (int hb = 0; hb < G::NHB; ++hb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)(acc[hb][q4 * 4 + e] * osc);
          *reinterpret_cast<bf16x4*>(row + hb * 32 + q4 * 8 + hf * 4) = v;
        }
    } else {      // this split's share, fp32; attn_dkv_reduce_kernel adds the splits up in a fixed order
      float* row = a.dkv_part + (((int64_t)sp * a.b + ib) * a.s + key) * (2 * dkv) + g * HD + (role ? 0 : dkv);
#pragma unroll
      for (int hb = 0; hb < G::NHB; ++hb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[hb][q4 * 4 + e] * osc;
          *reinterpret_cast<f32x4*>(row + hb * 32 + q4 * 8 + hf * 4) = v;
        }
    }
  }
}

// dK | dV of dqkv = sum over splits, in split order (bit-reproducible), rounded once to bf16
__global__ __launch_bounds__(256) void attn_dkv_reduce_kernel(AttnArgs a, int nsplit, int d, int dkv) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;       // one 4-column piece of one row
  const int per_row = 2 * dkv / 4;
  const int64_t rows = (int64_t)a.b * a.s;
  if (i >= rows * per_row) return;
  const int64_t row = i / per_row;
  const int c = (int)(i % per_row) * 4;
  f32x4 acc = *reinterpret_cast<const f32x4*>(a.dkv_part + row * (2 * dkv) + c);
  for (int sp = 1; sp < nsplit; ++sp) acc += *reinterpret_cast<const f32x4*>(a.dkv_part + ((int64_t)sp * rows + row) * (2 * dkv) + c);
  bf16x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = (bf16)acc[e];
  *reinterpret_cast<bf16x4*>((bf16*)a.dqkv + row * a.ld + d + c) = o;
}

// dynamic LDS of the kernels above
template <int HD> constexpr size_t fwd_lds() { return (size_t)4 * Geo<HD>::TILEB; }
template <int HD, int TQ> constexpr size_t dkv_lds() { return (size_t)2 * (2 * TQ * Geo<HD>::ROWB + 2 * TQ * 4) + (TQ / 32) * 4096 + 64; }   // + P slots and counts

template <typename K>
hipError_t allow_lds(K kern, size_t bytes) {
  return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// The dispatch rules below count workgroups against the CUs of a 256-CU chip (two resident 4-wavefront workgroups per
// CU for forward, dQ and the small dK/dV tile; the 8-wavefront ones sit one to a CU); the scratch size of the backward
// depends on them, so they use the constant rather than the device's count.
constexpr int64_t RESIDENT = 2 * 256;

// Forward / dQ workgroup shape: 8 wavefronts x 32 queries when that gives two workgroups per CU (they read every K/V
// tile once for twice the queries); else 4 x 32 queries; else (still under two per CU) 64 queries with the key range of
// each query block split over two wavefronts.
enum FwdShape { SHAPE_WIDE = 1, SHAPE_NARROW = 2, SHAPE_SPLIT = 3 };
static int64_t fwd_count(const AttnArgs& a, int bq) { return (int64_t)a.b * a.h * ((a.s + bq - 1) / bq); }
static FwdShape fwd_shape(const AttnArgs& a) {
  if (a.width >= 1 && a.width <= 3) return (FwdShape)a.width;
  if (fwd_count(a, fwd_bq(FWD_WIDE)) >= RESIDENT) return SHAPE_WIDE;
  if (fwd_count(a, fwd_bq(FWD_NARROW)) >= RESIDENT) return SHAPE_NARROW;
  return SHAPE_SPLIT;
}

template <int HD, int NT, int KS>
hipError_t fwd_launch(const AttnArgs& a, hipStream_t s) {
  static const hipError_t ready = allow_lds(attn_fwd_kernel<HD, NT, KS>, fwd_lds<HD>());
  if (ready != hipSuccess) return ready;
  const int nqt = (a.s + fwd_bq(NT, KS) - 1) / fwd_bq(NT, KS);
  // 4-wavefront workgroups sit two to a CU: when the whole grid is resident at once, pair heavy with light.  (8-wavefront
  // ones sit one to a CU and come in two rounds or more: heaviest first, and the light ones fill in behind.)
  const int fold = NT == FWD_NARROW && a.causal && (int64_t)a.b * a.h * nqt <= RESIDENT;
  hipLaunchKernelGGL((attn_fwd_kernel<HD, NT, KS>), dim3(a.h, nqt * a.b), dim3(NT), fwd_lds<HD>(), s, a, fold);
  return hipGetLastError();
}
template <int HD>
hipError_t fwd_t(const AttnArgs& a, hipStream_t s) {
  switch (fwd_shape(a)) {
    case SHAPE_WIDE: return fwd_launch<HD, FWD_WIDE, 1>(a, s);
    case SHAPE_NARROW: return fwd_launch<HD, FWD_NARROW, 1>(a, s);
    default: return fwd_launch<HD, FWD_NARROW, 2>(a, s);
  }
}

template <int HD, int NT, int KS>
hipError_t dq_launch(const AttnArgs& a, hipStream_t s) {
  static const hipError_t ready = allow_lds(attn_dq_kernel<HD, NT, KS>, fwd_lds<HD>());
  if (ready != hipSuccess) return ready;
  const int nqt = (a.s + fwd_bq(NT, KS) - 1) / fwd_bq(NT, KS);
  const int fold = NT == FWD_NARROW && a.causal && (int64_t)a.b * a.h * nqt <= RESIDENT;      // as in the forward
  hipLaunchKernelGGL((attn_dq_kernel<HD, NT, KS>), dim3(a.h, nqt * a.b), dim3(NT), fwd_lds<HD>(), s, a, fold);
  return hipGetLastError();
}

// Split a KV head's query heads over workgroups until the dK/dV grid has two workgroups per CU (or every query head
// has its own workgroup); the count must divide the group size.
static int dkv_splits(int b, int s, int h, int hkv, int tq) {
  const int grp = h / hkv;
  const int64_t wgs = (int64_t)b * hkv * ((s + tq - 1) / tq);
  int ns = 1;
  while (ns < grp && wgs * ns < RESIDENT) {
    int nx = ns + 1;
    while (grp % nx) ++nx;
    ns = nx;
  }
  return ns;
}
// 64-key workgroups when 128-key ones, split as far as they go, still number fewer than two per CU
static bool dkv_small(int b, int s, int h, int hkv, int width) {
  if (width) return width == 3;
  return (int64_t)b * hkv * ((s + DKV_TQ - 1) / DKV_TQ) * dkv_splits(b, s, h, hkv, DKV_TQ) < RESIDENT;
}

template <int HD, int TQ>
hipError_t dkv_launch(const AttnArgs& a, hipStream_t s) {
  constexpr size_t lds_bytes = dkv_lds<HD, TQ>();
  static const hipError_t ready = allow_lds(attn_dkv_kernel<HD, TQ>, lds_bytes);
  if (ready != hipSuccess) return ready;
  const int nsplit = a.dkv_part ? dkv_splits(a.b, a.s, a.h, a.hkv, TQ) : 1;
  const int nkt = (a.s + TQ - 1) / TQ;
  // two 64-key workgroups share a CU: when all are resident at once, pair heavy key tiles with light ones
  const int fold = TQ == DKV_TQ_SMALL && a.causal && (int64_t)a.b * a.hkv * nsplit * nkt <= RESIDENT;
  hipLaunchKernelGGL((attn_dkv_kernel<HD, TQ>), dim3(a.hkv * nsplit, nkt * a.b), dim3(TQ * 4), lds_bytes, s, a, nsplit, fold);
  if (nsplit > 1) {
    const int64_t pieces = (int64_t)a.b * a.s * (2 * a.hkv * HD / 4);
    hipLaunchKernelGGL(attn_dkv_reduce_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, s, a, nsplit, a.h * HD, a.hkv * HD);
  }
  return hipGetLastError();
}

template <int HD>
hipError_t bwd_t(const AttnArgs& a, hipStream_t s) {
  hipError_t e;      // dQ first: it also leaves delta = rowsum(dO * O) in a.delta for the dK/dV pass
  switch (fwd_shape(a)) {
    case SHAPE_WIDE: e = dq_launch<HD, FWD_WIDE, 1>(a, s); break;
    case SHAPE_NARROW: e = dq_launch<HD, FWD_NARROW, 1>(a, s); break;
    default: e = dq_launch<HD, FWD_NARROW, 2>(a, s); break;
  }
  if (e != hipSuccess) return e;
  return dkv_small(a.b, a.s, a.h, a.hkv, a.width) ? dkv_launch<HD, DKV_TQ_SMALL>(a, s) : dkv_launch<HD, DKV_TQ>(a, s);
}

}  // namespace

// Scratch of the backward: the fp32 partial dK | dV of every split.  Sized for either tile of the dK/dV kernel (the
// tile is chosen from the shape, or forced by AttnArgs::width).
int attn_bwd_splits(int b, int s, int h, int hkv) {
  const int n128 = dkv_splits(b, s, h, hkv, DKV_TQ), n64 = dkv_splits(b, s, h, hkv, DKV_TQ_SMALL);
  return n128 > n64 ? n128 : n64;
}
size_t attn_bwd_part_bytes(int b, int s, int h, int hkv, int hd) {
  const int ns = attn_bwd_splits(b, s, h, hkv);
  return ns > 1 ? (size_t)ns * b * s * 2 * hkv * hd * sizeof(float) : 0;
}

bool attn_mfma_supported(const AttnArgs& a) {
  if (a.hd != 64 && a.hd != 128) return false;
  if (a.ld % 8 || ((uintptr_t)a.qkv & 15) || ((uintptr_t)a.o & 15)) return false;
  if (a.dout && (((uintptr_t)a.dout & 15) || ((uintptr_t)a.dqkv & 15))) return false;
  if ((int64_t)a.s * a.ld * 2 >= ((int64_t)1 << 31)) return false;   // tile loads use 32-bit byte offsets inside a sequence
  if ((int64_t)a.b * ((a.s + 63) / 64) > 65535) return false;        // grid.y = tiles of a sequence x sequences, smallest tile
  return a.b > 0 && a.s > 0 && a.h > 0 && a.hkv > 0 && a.h % a.hkv == 0;
}

hipError_t attn_fwd_mfma(const AttnArgs& a, hipStream_t s) { return a.hd == 128 ? fwd_t<128>(a, s) : fwd_t<64>(a, s); }
hipError_t attn_bwd_mfma(const AttnArgs& a, hipStream_t s) { return a.hd == 128 ? bwd_t<128>(a, s) : bwd_t<64>(a, s); }

}  // namespace stg
