// bf16 MFMA GEMM for gfx950, the three operand layouts of a linear layer's
// forward, input-gradient and weight-gradient products (paper Appendix B):
//
//   NN  C[M,N]  = A[M,K] . B[K,N] (+ R)        forward,  A.W
//   NT  C[M,N]  = A[M,K] . B[N,K]^T            dgrad,    dZ.W^T
//   TN  C[M,N] += A[K,M]^T . B[K,N]   (fp32)   wgrad,    A^T.dZ
//
// Design: 256x256x64 macro tile per workgroup, 8 wavefronts (2x4, two per SIMD),
// each owning a 128x64 sub-tile as 8x4 v_mfma_f32_16x16x32_bf16 accumulators
// (128 fp32 registers per lane; on random data this MFMA shape sustains a higher
// rate than 32x32x16 -- the chip is power-limited there and it moves half as many
// accumulator registers per flop).  Operand tiles travel global -> LDS directly
// (buffer loads with the LDS bit: no staging registers, no ds_write instructions,
// hardware range check gives the zero fill at the edges) into a ring of five
// 32 KiB slots that the A and B tiles of the reduction take in turn: one barrier
// per K tile, loads issued at an even rate of one operand tile per k-step, a few
// MFMAs apart, each with at least half a K tile's time to land; fragments are
// double-buffered in registers and the loop body is an explicit two-stage
// software pipeline without branches.  Such a load writes each wavefront's
// 64 x 16 bytes to consecutive LDS addresses, so the tiles are unpadded and bank
// conflicts are avoided by choosing WHICH 16-byte piece each lane fetches (an XOR
// swizzle of the piece index).  An operand whose reduction index is contiguous in
// memory sits in LDS as [row][k] and is read with 16-byte loads; an operand whose
// reduction index is the slow one sits as [k][row] and is read with
// ds_read_b64_tr_b16, the LDS transpose load, so no layout needs a transposing
// copy.  The MFMA is issued with the operands swapped (computes the transposed
// 16x16 block), which leaves every lane with 4 consecutive columns of one row:
// 8-byte bf16 / 16-byte fp32 epilogue accesses.  Workgroup ids are remapped so
// that each XCD (own L2) works on a compact band of tiles.  A 128x256 half-height
// tile (4 wavefronts) takes over where full tiles would keep at most half of the
// CUs busy: the last round of a product, or a product with few tiles.
#include "common.h"
#include <type_traits>

namespace stg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = BM * BK * 2;                      // one operand tile, either layout: 32 KiB
constexpr size_t LDS_BYTES = (size_t)5 * TILE_BYTES;         // 160 KiB: the ring of operand tiles (five full-size slots)
static_assert(BM == BN, "both operand tiles share one geometry");

enum Epi { EPI_STORE = 0, EPI_RESID = 1, EPI_ACC32 = 2, EPI_GELU = 3, EPI_SWIGLU = 4, EPI_DGELU = 5, EPI_DSWIGLU = 6 };
// EPI_SWIGLU: a tile covers GLU_BN features j and holds, side by side in 32-column blocks, the gate columns j and
// the up columns f + j of the product (even blocks gate, odd blocks up), so that a lane's two accumulator blocks are
// the gate and the up value of the same 32 features and silu(gate) * up is formed in registers.
constexpr int GLU_BN = 128;

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char;
constexpr unsigned OOB = 0x80000000u;   // any offset >= num_records makes a buffer load return zeros

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// LDS placement of a tile's 16-byte pieces ("slots", slot s at byte 16*s):
//   [row][k] layout (KC, reduction index contiguous in memory): row r = 8 pieces; piece c (8 k's) of row r sits in
//     slot 8*r + (c ^ ((r >> 1) & 7)).  A fragment read takes piece c of 16 consecutive rows per quarter-wave, which
//     hit 16 different 16-byte bank groups.
//   [k][row] layout: reduction row k = 32 pieces of 8 rows; piece p sits in slot 32*k + (p ^ swz(k)),
//     swz(k) = ((k & 3) << 2) | (((k >> 3) & 1) << 1).  A transpose read by 16 lanes takes 32 bytes from each of 4
//     consecutive k rows, which land in 4 different 64-byte bank groups; the next 16 lanes read 8 rows further on,
//     which the second term moves to the other 32 bytes of those groups.
// Per-thread global byte offsets at k = 0 of the pieces it fetches: load j of wavefront w fills slots
// (j*8 + w)*64 .. +63, lane l the l-th of them.  Rows past the end of the matrix fall outside the buffer's range
// by themselves or are redirected to OOB, which stores zeros.
// (a [row][k] tile may have any multiple of 8 rows: WAVES * 64 * CH pieces; a [k][row] tile has PCS pieces = 8 * PCS rows
// per reduction row, 32 or 16, and the same formulas with 32 replaced by PCS)
// glu_f > 0 (a [k][row] B tile of EPI_SWIGLU): row0 is the tile's first feature and piece p = 8 columns of block p / 4
// fetches columns (odd block ? glu_f : 0) + row0 + (p / 8) * 32 + (p % 4) * 8 ..
template <bool KC, int WAVES, int CH, int PCS = 32>
__device__ __forceinline__ void tile_offsets(unsigned (&off)[CH], int64_t ld, int row0, int rows, int wave, int lane,
                                             int glu_f = 0) {
  static_assert(KC || WAVES * 64 * CH == BK * PCS, "every 16-byte piece of the tile has one owner");
#pragma unroll
  for (int j = 0; j < CH; ++j) {
    const int s = (j * WAVES + wave) * 64 + lane;
    if (KC) {
      const int r = s >> 3, c = (s & 7) ^ ((r >> 1) & 7);
      off[j] = row0 + r < rows ? (unsigned)(((int64_t)(row0 + r) * ld + c * 8) * 2) : OOB;
    } else {
      const int k = s / PCS, p = (s % PCS) ^ (((k & 3) << 2) | (((k >> 3) & 1) << 1));
      int row = row0 + p * 8;
      bool ok = row < rows;
      if (glu_f) {
        const int feat = row0 + (p >> 3) * 32 + (p & 3) * 8;
        ok = feat < glu_f;
        row = ((p >> 2) & 1) ? glu_f + feat : feat;
      }
      off[j] = ok ? (unsigned)(((int64_t)k * ld + row) * 2) : OOB;
    }
  }
}

// one operand tile at reduction offset k0 (a multiple of BK; K % BK == 0 for a KC operand): global -> LDS, no
// registers, no branches.  OOB + anything below 2 GiB stays out of range; reduction rows >= K of a non-KC operand
// are past the end of the buffer.  `wave` must be wave-uniform (the LDS address of such a load is a scalar).
//
// The load is written as inline assembly on purpose: with the builtin, the compiler cannot tell these LDS writes
// from the fragment reads of the other buffer and drains the vector-memory counter before the next LDS read, which
// serialises every K tile on the full memory latency.  Completion is awaited by hand (vmcnt(0) before the barrier
// that publishes the tile).  m0 carries the wavefront's LDS destination; lane l lands at m0 + 16*l.  Nothing else in
// this kernel uses m0, which the compiler reserves and re-materialises before each use of its own.
typedef int rsrc_words __attribute__((ext_vector_type(4)));
__device__ __forceinline__ rsrc_words raw_rsrc(const void* base, unsigned bytes) {
  const uint64_t a = (uint64_t)base;
  return rsrc_words{(int)(unsigned)a, (int)(unsigned)((a >> 32) & 0xffffu), (int)bytes, 0x00020000};
}
__device__ __forceinline__ void load_to_lds_b128(rsrc_words rsrc, unsigned lds_addr, unsigned voffset) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(voffset), "s"(rsrc) : "memory");
}
template <bool KC, int WAVES, int CH>
__device__ __forceinline__ void g2s_one(lds_char* tile, rsrc_words rsrc, const unsigned (&off)[CH], int64_t ld, int k0,
                                        int wave, int j) {
  const unsigned step = KC ? (unsigned)k0 * 2u : (unsigned)((int64_t)k0 * ld * 2);
  load_to_lds_b128(rsrc, (unsigned)(size_t)(tile + (j * WAVES + wave) * 1024), off[j] + step);
}
template <bool KC, int WAVES, int CH>
__device__ __forceinline__ void g2s(lds_char* tile, rsrc_words rsrc, const unsigned (&off)[CH], int64_t ld, int k0, int wave) {
#pragma unroll
  for (int j = 0; j < CH; ++j) g2s_one<KC, WAVES, CH>(tile, rsrc, off, ld, k0, wave, j);
}

// Per-lane LDS byte offsets (inside one operand tile) from which the fragments of a 16-row block are read.
// Fragment = 16(row) x 32(k): lane l holds row l%16, k = (l/16)*8 .. +7.
//   KC:  ad[ks], ks = k-step 0..1; block b of 16 rows adds 2048 bytes (the swizzle repeats every 16 rows)
//   else ad[b], b = 16-row block index counted from row0; k-step ks adds 32 reduction rows of PCS * 16 bytes; the
//        transpose load: in a 16-lane group, lane i addresses row (i/4) of a 4(k) x 16(row) block at column 4*(i%4)
//        and receives column i of the block, i.e. 4 consecutive k for its own row; the four groups of a wavefront
//        take the reduction rows g*8 .. g*8+3 (and, in a second load, 4 rows further on)
template <bool KC, int NB, int PCS = 32>
__device__ __forceinline__ void frag_offsets(unsigned (&ad)[NB], int row0, int lane) {
  if (KC) {
    const int r = row0 + (lane & 15), sw = (r >> 1) & 7, h = lane >> 4;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) ad[ks] = (unsigned)((r * 8 + ((4 * ks + h) ^ sw)) * 16);
  } else {
    const int g = lane >> 4, li = lane & 15;
    const int krow = g * 8 + (li >> 2);
    const int sw = ((krow & 3) << 2) | (((krow >> 3) & 1) << 1);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int p = ((row0 >> 4) + b) * 2 + ((li & 3) >> 1);                   // 16-byte piece of the reduction row
      ad[b] = (unsigned)(krow * (PCS * 16) + (p ^ sw) * 16 + (li & 1) * 8);
    }
  }
}

// `pt`: the tile's LDS address plus the offsets above
template <bool KC, int NB, int PCS = 32>
__device__ __forceinline__ bf16x8 frag(lds_char* const (&pt)[NB], int b, int ks) {
  if (KC) {
    return *reinterpret_cast<__attribute__((address_space(3))) const bf16x8*>(pt[ks] + b * 2048);
  } else {
    typedef s16x4 __attribute__((address_space(3))) * lds_p;
    lds_char* p = pt[b] + ks * (32 * PCS * 16);
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 4 * PCS * 16));
    union { struct { s16x4 a, b; } s; bf16x8 v; } u;
    u.s.a = lo; u.s.b = hi;
    return u.v;
  }
}

// TN = 32-column groups per wavefront: 2 -> 8 wavefronts of 128x64 (two per SIMD, 128 accumulator registers each),
// 4 -> 4 wavefronts of 128x128 (one per SIMD, 256 accumulator registers, a third less LDS read traffic)
// K segments: the reduction may run over `nseg` operand pairs of equal shape, pair s being (A, B) moved by
// seg_delta[s] bytes (seg_delta[0] == 0): C (+)= sum_s A_s . B_s with the K tiles taken in order s = 0, 1, ...  One
// pass over K then does the work of nseg launches with a single read-modify-write of C, and -- fp32 accumulators
// written to and read back from fp32 memory unchanged -- gives the same bits as those launches one after another.
// WR, WC = rows and columns of 128 in the tile: (2, 2) -> 256 x 256 (wave grid 2 x WGN); (1, 2) -> 128 x 256 (wave grid
// 1 x WGN, half the wavefronts); (1, 1) -> 128 x 128 (four wavefronts of 64 x 64); A must be a [row][k] operand unless
// the tile is a full one.  The smaller tiles exist for the work a grid of full tiles would leave to a fraction of the
// CUs: the last, partly filled round of a product, and products with few tiles.
template <bool AKC, bool BKC, int EPI, int TN, int WR = 2, int WC = 2>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, int m0, int n0, lds_char* smem, int nseg = 1,
                                          const int64_t* seg_delta = nullptr) {
  static_assert(WR == 2 || (WR == 1 && AKC), "the smaller tiles take a [row][k] A operand");
  static_assert(WC == 2 || (WR == 1 && TN == 2 && (EPI == EPI_STORE || EPI == EPI_RESID)), "the 128 x 128 tile: plain epilogues only");
  constexpr bool GLU = EPI == EPI_SWIGLU;
  static_assert(!GLU || (TN == 2 && !BKC), "gate and up blocks are the two halves of a wavefront's columns");
  constexpr int BMV = WR * 128, BNV = WC * 128;                                    // tile: BMV rows, BNV columns
  constexpr int RW = WC == 1 ? 64 : 128;                                           // rows of a wavefront's sub-tile
  constexpr int WGN = BNV / (TN * 32), WAVES = (BMV / RW) * WGN;
  constexpr int A_BYTES = BMV * BK * 2, B_BYTES = BNV * BK * 2;
  constexpr int PCS = BNV / 8;                                                     // 16-byte pieces per row of C / per reduction row of a [k][row] B tile
  constexpr int CHA = (A_BYTES / 16) / (WAVES * 64), CHB = (B_BYTES / 16) / (WAVES * 64); // loads per thread and K tile
  constexpr int NI = RW / 16, NJ = 2 * TN;                                         // 16 x 16 accumulator blocks per wavefront
  // The ring of operand tiles (see below): DEPTH K tiles ahead of the one being multiplied, 2 * DEPTH + 1 slots.  The
  // 128 x 128 tile's operand tiles are half the size and its K tile takes a quarter of the MFMA time, so the same LDS
  // holds -- and the same lead in time needs -- twice the depth: with a lead of two K tiles (about 1 us here) operands
  // that come from HBM rather than from a cache arrive late, and products of this tile ran a quarter to a third slower
  // on cold operands than on warm ones.
  constexpr bool SMALL = WR == 1 && WC == 1;
  constexpr int SLOT = SMALL ? TILE_BYTES / 2 : TILE_BYTES, DEPTH = SMALL ? 4 : 2, NSLOT = 2 * DEPTH + 1;
  static_assert(A_BYTES <= SLOT && B_BYTES <= SLOT && (size_t)NSLOT * SLOT <= LDS_BYTES, "ring fits");
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = (wave / WGN) * RW, wn = (wave % WGN) * (TN * 32);

  // buffer descriptors cover exactly the rows that exist: KC operand = [rows, ld], other = [K, ld]
  const unsigned bytesA = (unsigned)(((int64_t)((AKC ? g.M : g.K) - 1) * g.lda + (AKC ? g.K : g.M)) * 2);
  const unsigned bytesB = (unsigned)(((int64_t)((BKC ? g.N : g.K) - 1) * g.ldb + (BKC ? g.K : g.N)) * 2);
  rsrc_words rsA = raw_rsrc(g.A, bytesA), rsB = raw_rsrc(g.B, bytesB);
  unsigned offa[CHA], offb[CHB];
  tile_offsets<AKC, WAVES, CHA>(offa, g.lda, m0, g.M, wave, lane);
  tile_offsets<BKC, WAVES, CHB, PCS>(offb, g.ldb, n0, g.N, wave, lane, GLU ? g.N / 2 : 0);

  // LDS map: a ring of NSLOT slots of one operand tile each; the operand tiles of the reduction take the slots in the
  // order A0 B0 A1 B1 A2 ..., tile number i (A_t = 2t, B_t = 2t + 1) sitting in slot i % NSLOT.
  const int nk = ((g.K + BK - 1) / BK) * nseg;
  // where the next tile of each operand to fetch lies: segment and reduction offset inside it (all wave-uniform)
  int segA = 0, kA = 0, segB = 0, kB = 0;
  // reduction offset at which an operand moves on to its next segment (never, in the last one): one compare per K tile,
  // its branch laid out as not taken -- a taken branch costs the single wavefront of a SIMD, and with it the SIMD's MFMA
  // pipe, some twenty cycles
  constexpr int NEVER = 0x7fffffff;
  int endA = (EPI == EPI_ACC32 && nseg > 1) ? g.K : NEVER, endB = endA;
  auto advanceA = [&]() {
    kA += BK;
    if (EPI == EPI_ACC32 && __builtin_expect(kA >= endA, 0)) {
      kA = 0; ++segA; rsA = raw_rsrc((const char*)g.A + seg_delta[segA], bytesA);
      if (segA + 1 >= nseg) endA = NEVER;
    }
  };
  auto advanceB = [&]() {
    kB += BK;
    if (EPI == EPI_ACC32 && __builtin_expect(kB >= endB, 0)) {
      kB = 0; ++segB; rsB = raw_rsrc((const char*)g.B + seg_delta[segB], bytesB);
      if (segB + 1 >= nseg) endB = NEVER;
    }
  };
  // start-up: A0 B0 A1 B1 ... of the first DEPTH K tiles, as far as they exist
#pragma unroll
  for (int t = 0; t < DEPTH; ++t)
    if (t == 0 || nk > t) {
      g2s<AKC, WAVES, CHA>(smem + 2 * t * SLOT, rsA, offa, g.lda, kA, wave);
      advanceA();
      g2s<BKC, WAVES, CHB>(smem + (2 * t + 1) * SLOT, rsB, offb, g.ldb, kB, wave);
      advanceB();
    }

  // acc[i][j][e] = C[m0 + wm + i*16 + lane%16][n0 + wn + j*16 + (lane/16)*4 + e]: the MFMA is issued with the operands
  // swapped, which leaves every lane with 4 consecutive columns of one row.
  // Accumulators start at zero, or -- weight gradients, C += A^T.B -- at the current value of C: the read half of
  // the read-modify-write then travels together with the first operand tiles instead of stalling the epilogue.
  const int row_l = lane & 15, col_l = (lane >> 4) * 4;
  f32x4 acc[NI][NJ];
  if (EPI == EPI_ACC32) {
    const __amdgpu_buffer_rsrc_t rsC = make_rsrc(g.C, (unsigned)(((int64_t)(g.M - 1) * g.ldc + g.N) * 4));
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int m = m0 + wm + i * 16 + row_l;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int n = n0 + wn + j * 16 + col_l;
        const unsigned off = (m < g.M && n < g.N) ? (unsigned)(((int64_t)m * g.ldc + n) * 4) : OOB;
        acc[i][j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsC, (int)off, 0, 0));
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // fragment addresses in the slots being read
  constexpr int NPA = AKC ? 2 : NI, NPB = BKC ? 2 : NJ;
  lds_char *pa[NPA], *pb[NPB];
  {
    unsigned ada[NPA], adb[NPB];
    frag_offsets<AKC, NPA>(ada, wm, lane);
    frag_offsets<BKC, NPB, PCS>(adb, wn, lane);
#pragma unroll
    for (int x = 0; x < NPA; ++x) pa[x] = smem + ada[x];
#pragma unroll
    for (int x = 0; x < NPB; ++x) pb[x] = smem + SLOT + adb[x];
  }
  int slotA = 0;               // slot of the A tile being read; its B tile sits in the next slot of the ring

  // Software pipeline, one K tile (2 k-steps of 32) per trip t, fragments double-buffered in registers:
  //   S0  MFMA k0 | read frags k1 | A(t+2)'s loads
  //   -- wait for A(t+1), B(t+1); barrier --
  //   S1  MFMA k1 | frags k0 of tile t+1 | B(t+2)'s loads
  // The barrier frees the two slots just read: B(t+2) goes into A(t)'s, A(t+3) -- half a trip later -- into B(t)'s.
  // With five slots the loads are issued at an even rate, one operand tile per k-step and a few MFMAs apart, instead of
  // all at once after the barrier (the CU's vector-memory path takes about half a trip to move a trip's 64 KiB, and a
  // wavefront whose load does not fit the queue stands still, MFMAs included), and every load has half a trip or more
  // to land.  Away from the end of the reduction the loop body has no branches.
  constexpr int NMFMA = NI * NJ;                                // MFMAs per k-step
  constexpr int NFRAG = NI + NJ;                                // fragments per k-step
  static_assert(NMFMA % CHA == 0 && NMFMA % CHB == 0 && NMFMA >= 2 * NFRAG, "placement of loads and fragment reads");
  bf16x8 fa[2][NI], fb[2][NJ];
  // one k-step: the MFMAs on fragment set `cur`; after every second MFMA one fragment of `ks_next` into the other set
  // (B's first: the first MFMAs of the next k-step need all of them); and the loads of operand tile `op` (0 = A, 1 = B)
  // spread between the MFMAs
  auto kstep = [&](auto cur_c, auto ks_c, auto op_c, auto tail_c, lds_char* dst) __attribute__((always_inline)) {
    constexpr int cur = decltype(cur_c)::value, ks_next = decltype(ks_c)::value, op = decltype(op_c)::value;
    constexpr int NL = op ? CHB : CHA, GAP = NMFMA / NL;
    constexpr bool do_load = !decltype(tail_c)::value;            // the last DEPTH trips have nothing left to fetch
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int js = (TN == 2 && (i & 1)) ? NJ - 1 - j : j;     // boustrophedon: consecutive MFMAs always share one operand
                                                                  // (with four column groups the register allocator spills on it)
        acc[i][js] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[cur][js], fa[cur][i], acc[i][js], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        const int n = i * NJ + j;
        if (n % 2 == 0 && n / 2 < NFRAG) {
          const int f = n / 2;
          if (f < NJ) fb[cur ^ 1][f] = frag<BKC, NPB, PCS>(pb, f, ks_next);
          else fa[cur ^ 1][f - NJ] = frag<AKC, NPA>(pa, f - NJ, ks_next);
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (do_load) if (n % GAP == GAP - 1) {
          const int l = n / GAP;
          if (op == 0) g2s_one<AKC, WAVES, CHA>(dst, rsA, offa, g.lda, kA, wave, l);
          else g2s_one<BKC, WAVES, CHB>(dst, rsB, offb, g.ldb, kB, wave, l);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
  };
  std::integral_constant<int, 0> c0; std::integral_constant<int, 1> c1;

  __builtin_amdgcn_s_waitcnt(0);   // the start-up tiles (and C for weight gradients) landed
  __syncthreads();
#pragma unroll
  for (int j = 0; j < NJ; ++j) fb[0][j] = frag<BKC, NPB, PCS>(pb, j, 0);
#pragma unroll
  for (int i = 0; i < NI; ++i) fa[0][i] = frag<AKC, NPA>(pa, i, 0);
  int kt = 0;
  auto trip = [&](auto tail_c) __attribute__((always_inline)) {
    constexpr bool tail = decltype(tail_c)::value;
    // ring position (wave-uniform) of tile 2(kt + DEPTH) = A(kt+DEPTH): the slot before A(kt)'s, which B(kt-1) has left;
    // tile 2(kt + DEPTH) + 1 = B(kt+DEPTH) takes A(kt)'s slot
    const int s4 = slotA == 0 ? NSLOT - 1 : slotA - 1;
    kstep(c0, c1, c0, tail_c, smem + s4 * SLOT);
    if (!tail) advanceA();
    // A(kt+1), B(kt+1) have landed once nothing older than the loads of A(kt+2) ... A(kt+DEPTH) is outstanding (in the
    // last trips: of the tiles that are left beyond kt+1); own LDS reads are done
    constexpr int VM = (DEPTH - 1) * CHA + (DEPTH - 2) * CHB;
    static_assert(VM < 64, "vmcnt is a 6-bit count");
    auto wait_vm = [](auto n_c) { constexpr int n = decltype(n_c)::value; __builtin_amdgcn_s_waitcnt(0x0070 | (n & 15) | ((n >> 4) << 14)); };
    if (!tail) wait_vm(std::integral_constant<int, VM>{});
    else if (DEPTH == 4 && nk - kt == 4) wait_vm(std::integral_constant<int, DEPTH == 4 ? 2 * (CHA + CHB) : 0>{});
    else if (DEPTH == 4 && nk - kt == 3) wait_vm(std::integral_constant<int, DEPTH == 4 ? CHA + CHB : 0>{});
    else __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    {
      const int dA = (slotA >= NSLOT - 2 ? 2 - NSLOT : 2) * SLOT;
      const int sB = slotA + 1 >= NSLOT ? slotA + 1 - NSLOT : slotA + 1;
      const int dB = (sB >= NSLOT - 2 ? 2 - NSLOT : 2) * SLOT;
#pragma unroll
      for (int x = 0; x < NPA; ++x) pa[x] += dA;
#pragma unroll
      for (int x = 0; x < NPB; ++x) pb[x] += dB;
    }
    kstep(c1, c0, c1, tail_c, smem + slotA * SLOT);           // (fragments past the last tile are read and not used)
    if (!tail) advanceB();
    slotA = slotA + 2 >= NSLOT ? slotA + 2 - NSLOT : slotA + 2;
  };
  for (; kt + DEPTH < nk; ++kt) trip(std::false_type{});
  for (; kt < nk; ++kt) trip(std::true_type{});

  // epilogue
  if (EPI != EPI_ACC32 && g.bias) {       // wave-uniform; the bias of a column goes to every row of it
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      int n = n0 + wn + j * 16 + col_l;
      bool ok = n < g.N;
      if (GLU) { const int feat = n0 + (wn >> 6) * 32 + (j & 1) * 16 + col_l; ok = feat < g.N / 2; n = (j >> 1) ? g.N / 2 + feat : feat; }
      if (ok) {
        const bf16x4 b = *reinterpret_cast<const bf16x4*>((const bf16*)g.bias + n);
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][e] += (float)b[e];
      }
    }
  }
  const int sub_b = (col_l & 4) * 2;      // byte inside a 16-byte piece at which this lane's 4 columns start
  if constexpr (EPI == EPI_DGELU || EPI == EPI_DSWIGLU) {
    // Activation backward on the fp32 accumulators (da), in place over the stashed z, in four quarters of the tile: a
    // quarter takes 32 rows from each 128-row half, so that every wavefront owns two of its accumulator block rows in
    // it.  The quarter's z columns (gate, and for SwiGLU up) come global -> LDS directly, whole rows (row r's piece p at
    // r*512 + ((p ^ (r & 31)) << 4), the up rows after the gate rows); the wavefronts rewrite their elements in LDS
    // (each element has one owner); everybody stores the rows back.  Two quarter buffers: the next quarter's loads are
    // in flight during this quarter's arithmetic and stores.
    constexpr int NOP = EPI == EPI_DSWIGLU ? 2 : 1;              // z operands per row: gate (| up)
    constexpr int QROWS = WR * 32;                               // staged rows per quarter
    constexpr int OPB = QROWS * 512, QBUF = NOP * OPB;           // bytes per operand and per quarter
    constexpr int NLD = (QROWS * 32) / (WAVES * 64);             // 16-byte pieces per thread, operand and quarter
    static_assert(NI == 8 && 2 * QBUF <= (int)LDS_BYTES, "quarters of two block rows per wavefront");
    const int f = g.N;
    const rsrc_words rsZ = raw_rsrc(g.Z, (unsigned)((((int64_t)(g.M - 1) * g.ldz) + NOP * f) * 2));
    typedef __attribute__((address_space(3))) bf16x4* lds_b4;
    auto quarter_loads = [&](int q, lds_char* buf) __attribute__((always_inline)) {
#pragma unroll
      for (int o = 0; o < NOP; ++o)
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
          const int s = (j * WAVES + wave) * 64 + lane, sr = s >> 5, p = (s & 31) ^ (sr & 31);
          const int row = m0 + (sr >> 5) * 128 + q * 32 + (sr & 31), col = n0 + p * 8;
          const unsigned off = (row < g.M && col < f) ? (unsigned)(((int64_t)row * g.ldz + o * f + col) * 2) : OOB;
          load_to_lds_b128(rsZ, (unsigned)(size_t)(buf + o * OPB + (j * WAVES + wave) * 1024), off);
        }
    };
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();                   // the main loop's last fragment reads are done: the ring is free
    quarter_loads(0, smem);
    quarter_loads(1, smem + QBUF);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      lds_char* buf = smem + (q & 1) * QBUF;
      __builtin_amdgcn_s_waitcnt(0);   // this quarter's rows (issued a quarter ago) and the previous quarter's stores
      __syncthreads();
#pragma unroll
      for (int ii = 0; ii < 2; ++ii) {
        const int i = 2 * q + ii;
        const int sr = (wm >> 7) * 32 + ii * 16 + row_l;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int p = (wn + j * 16 + col_l) >> 3;
          lds_char* at = buf + sr * 512 + ((p ^ (sr & 31)) << 4) + sub_b;
          if (EPI == EPI_DGELU) {
            bf16x4 u = *(lds_b4)at, o4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float uv = (float)u[e];
              const float dgl = 0.5f * (1.f + erff(uv * 0.70710678118654752f)) + uv * 0.39894228040143268f * __expf(-0.5f * uv * uv);
              o4[e] = (bf16)(acc[i][j][e] * dgl);
            }
            *(lds_b4)at = o4;
            __builtin_amdgcn_sched_barrier(0);
          } else {
            bf16x4 gt = *(lds_b4)at, up = *(lds_b4)(at + OPB), og, ou;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float gv = (float)gt[e], uv = (float)up[e], d = acc[i][j][e];
              const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-gv));
              og[e] = (bf16)(d * uv * (sg + gv * sg * (1.f - sg)));
              ou[e] = (bf16)(d * gv * sg);
            }
            *(lds_b4)at = og;
            *(lds_b4)(at + OPB) = ou;
          }
        }
      }
      __syncthreads();
#pragma unroll
      for (int o = 0; o < NOP; ++o)
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
          const int s = (j * WAVES + wave) * 64 + lane, sr = s >> 5, p = s & 31;      // lane order = column order: whole rows
          const int row = m0 + (sr >> 5) * 128 + q * 32 + (sr & 31), col = n0 + p * 8;
          const u32x4 v = *reinterpret_cast<__attribute__((address_space(3))) const u32x4*>(buf + o * OPB + sr * 512 + ((p ^ (sr & 31)) << 4));
          if (row < g.M && col < f) *reinterpret_cast<u32x4*>((bf16*)g.Z + (int64_t)row * g.ldz + o * f + col) = v;
        }
      if (q + 2 < 4) {
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): own reads of the buffer are done
        __syncthreads();                       // ... and everybody else's
        quarter_loads(q + 2, buf);
      }
    }
    return;
  }
  if (EPI == EPI_STORE || EPI == EPI_GELU || EPI == EPI_SWIGLU) {
    // bf16 output: the tile goes through LDS (128 KiB of what the operand ring held) so that the global stores are
    // whole rows of the tile (512 bytes; 256 for the 128-column tile), 16 bytes per lane, instead of 8-byte fragments of
    // 16 rows.  Row r's 16-byte piece p (of PCS) sits at r*PCS*16 + ((p ^ (r % PCS)) << 4): the fragment writes of 16
    // rows spread over all banks and a row is read back as a permutation of itself.  No loads are in flight here (none is issued past the last K tile); the barrier waits
    // for the other wavefronts' last fragment reads.
    // EPI_SWIGLU: pieces 0..15 of a staged row are the tile's 128 gate columns, pieces 16..31 its 128 up columns (two
    // 256-byte runs of the output row).
    const int glu_f = g.N / 2;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    auto stage_tile = [&](auto fn) {         // fn(acc) -> LDS as bf16, in the layout above
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int r = wm + i * 16 + row_l;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int p = GLU ? (j >> 1) * 16 + (wn >> 6) * 4 + (j & 1) * 2 + (col_l >> 3) : (wn + j * 16 + col_l) >> 3;
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16)fn(acc[i][j][e]);
          *reinterpret_cast<__attribute__((address_space(3))) bf16x4*>(smem + r * (PCS * 16) + ((p ^ (r & (PCS - 1))) << 4) + sub_b) = o;
          if (EPI == EPI_GELU) __builtin_amdgcn_sched_barrier(0);      // keeps the erf expansions from piling up in registers
        }
      }
    };
    auto store_tile = [&](bf16* out, int64_t ld) {      // LDS -> global, whole rows
      constexpr int RPI = 64 / PCS;                      // rows per instruction
      const int p = lane & (PCS - 1);
      int n = n0 + p * 8;
      bool n_ok = n < g.N;
      if (GLU) { const int feat = n0 + (p & 15) * 8; n_ok = feat < glu_f; n = (p >> 4) ? glu_f + feat : feat; }
#pragma unroll
      for (int t = 0; t < BMV / WAVES / RPI; ++t) {
        const int r = wave * (BMV / WAVES) + RPI * t + lane / PCS, m = m0 + r;
        const u32x4 v = *reinterpret_cast<__attribute__((address_space(3))) const u32x4*>(smem + r * (PCS * 16) + ((p ^ (r & (PCS - 1))) << 4));
        if (m < g.M && n_ok) *reinterpret_cast<u32x4*>(out + (int64_t)m * ld + n) = v;   // N % 8 == 0
      }
    };
    stage_tile([](float v) { return v; });
    __syncthreads();
    store_tile((bf16*)g.C, g.ldc);
    if (EPI == EPI_STORE) return;
    // the activation, from the fp32 accumulators
    __syncthreads();                  // every wavefront has read the staged z tile back
    if (EPI == EPI_GELU) {
      stage_tile([](float u) { return 0.5f * u * (1.f + erff(u * 0.70710678118654752f)); });
      __syncthreads();
      store_tile((bf16*)g.C2, g.ldc2);
    } else {
      // a = silu(gate) * up: 128 features per row = 256 bytes; rows with bit 4 set use the upper half of their
      // 512-byte LDS row so that rows r and r + 16 do not share banks
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const int r = wm + i * 16 + row_l;
#pragma unroll
        for (int jj = 0; jj < NJ / 2; ++jj) {
          const int fp = (wn >> 6) * 4 + jj * 2 + (col_l >> 3);
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float gv = acc[i][jj][e];
            o[e] = (bf16)(gv * __builtin_amdgcn_rcpf(1.f + __expf(-gv)) * acc[i][jj + NJ / 2][e]);
          }
          *reinterpret_cast<__attribute__((address_space(3))) bf16x4*>(smem + r * 512 + ((((r & 16) | fp) ^ (r & 15)) << 4) + sub_b) = o;
        }
      }
      __syncthreads();
      const int pc = lane & 15, feat = n0 + pc * 8;
#pragma unroll
      for (int t = 0; t < BMV / WAVES / 4; ++t) {
        const int r = wave * (BMV / WAVES) + 4 * t + (lane >> 4), m = m0 + r;
        const u32x4 v = *reinterpret_cast<__attribute__((address_space(3))) const u32x4*>(smem + r * 512 + ((((r & 16) | pc) ^ (r & 15)) << 4));
        if (m < g.M && feat < glu_f) *reinterpret_cast<u32x4*>((bf16*)g.C2 + (int64_t)m * g.ldc2 + feat) = v;
      }
    }
    return;
  }
  if constexpr (EPI == EPI_ACC32) {
    // acc already holds C + A^T.B.  Buffer stores like the loads that fetched C: one 32-bit offset per row block and
    // column block, elements outside the matrix redirected out of range and dropped -- no branch per store, which with
    // one wavefront per SIMD would hold up everything behind it
    const __amdgpu_buffer_rsrc_t rsC = make_rsrc(g.C, (unsigned)(((int64_t)(g.M - 1) * g.ldc + g.N) * 4));
    unsigned col_b[NJ];                // byte offset of the lane's columns inside a row; N % 8 == 0 and n % 4 == 0: the 4
                                       // columns are in or out together
#pragma unroll
    for (int j = 0; j < NJ; ++j) col_b[j] = (unsigned)(n0 + wn + j * 16 + col_l) * 4u;
    const unsigned row_b = (unsigned)((int64_t)(m0 + wm + row_l) * g.ldc * 4), step_b = (unsigned)g.ldc * 64u;   // 16 rows on
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const bool row_ok = m0 + wm + i * 16 + row_l < g.M;
      const unsigned base = row_b + (unsigned)i * step_b;       // (wraps only for rows that are not there)
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const bool ok = row_ok && n0 + wn + j * 16 + col_l < g.N;
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[i][j]), rsC, (int)(ok ? base + col_b[j] : OOB), 0, 0);
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int m = m0 + wm + i * 16 + row_l;
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int n = n0 + wn + j * 16 + col_l;
      if (n >= g.N) continue;          // N % 8 == 0 and n % 4 == 0: the 4 columns are in or out together
      f32x4 v = acc[i][j];
      {
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

// Walk order of the 256x256 tiles of one product: groups of 8 tile rows, column by column inside a group.
__device__ __forceinline__ void tile_of(int idx, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
  constexpr int GROUP = 8;
  const int in_group = GROUP * tiles_n;
  const int gid = idx / in_group;
  const int first_m = gid * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  tile_m = first_m + (idx % in_group) % gsz;
  tile_n = (idx % in_group) / gsz;
}

// one workgroup per tile: workgroup `bid` takes the full tile number first + bid of the walk order (WR == 2), or the
// upper (even bid) / lower (odd bid) 128 rows of full tile number first + bid / 2 (WR == 1)
template <bool AKC, bool BKC, int EPI, int TN, int WR>
// The second launch bound (wavefronts per SIMD the register budget must allow) is 2 for the half-height tile: its four
// wavefronts of 128 x 64 then get the 256 registers the full tile's eight have, all of them ordinary VGPRs.  Left at
// one per SIMD (512 registers), the compiler kept the accumulators in AGPRs, gave the MFMAs a destination other than
// their C operand and moved 128-190 registers between the two files on every trip of the main loop.
__global__ __launch_bounds__(WR * 512 / TN, WR == 1 ? 2 : 1) void gemm_mfma_kernel(GemmArgs g, int tiles_m, int tiles_n, int first) {
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  // XCD-aware tile order: consecutive workgroup ids go to different XCDs, so give XCD x the
  // x-th contiguous band of the tile sequence.
  int bid = blockIdx.x;
  const int nb = gridDim.x;
  {
    const int per = nb >> 3, main = per << 3;
    if (bid < main) bid = (bid & 7) * per + (bid >> 3);
  }
  int tile_m, tile_n;
  tile_of(first + (WR == 2 ? bid : bid >> 1), tiles_m, tiles_n, tile_m, tile_n);
  gemm_tile<AKC, BKC, EPI, TN, WR>(g, tile_m * BM + (WR == 2 ? 0 : (bid & 1) * 128), tile_n * (EPI == EPI_SWIGLU ? GLU_BN : BN),
                                   (lds_char*)smem_raw);
}

// one workgroup per 128 x 128 tile (four wavefronts of 64 x 64): workgroup `bid` takes quadrant bid % 4 of the full
// tile number first + bid / 4 of the walk order; a quadrant that lies outside the matrix has nothing to do
template <bool AKC, bool BKC, int EPI>
__global__ __launch_bounds__(256, 2) void gemm_quarter_kernel(   // (register budget: as for the half-height tile)
    GemmArgs g, int tiles_m, int tiles_n, int first) {
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  int bid = blockIdx.x;
  {
    const int per = (int)gridDim.x >> 3, main = per << 3;
    if (bid < main) bid = (bid & 7) * per + (bid >> 3);
  }
  int tile_m, tile_n;
  tile_of(first + (bid >> 2), tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM + (bid & 1) * 128, n0 = tile_n * BN + ((bid >> 1) & 1) * 128;
  if (m0 >= g.M || n0 >= g.N) return;                  // the same for the whole workgroup
  gemm_tile<AKC, BKC, EPI, 2, 1, 1>(g, m0, n0, (lds_char*)smem_raw);
}

// Several weight-gradient products C_p += A_p^T . B_p in one launch of persistent workgroups.  Each workgroup
// takes the tiles  r * gridDim.x + (its slot)  of the concatenated tile list, r = 0, 1, ...: after it has issued a
// tile's stores it goes straight on to the next tile's C and operand loads, so the read-modify-write of the fp32
// gradients -- a quarter of such a product's time when all workgroups do it at once and then wait -- overlaps
// with MFMA work.  Every C tile is still produced by one workgroup in one pass over K: results are bit-identical
// to separate launches.
constexpr int GROUP_MAX = 16;
struct GemmGroup {
  int n, total_tiles, nseg;
  int first_tile[GROUP_MAX + 1];
  int64_t seg_delta[GEMM_MAX_SEG];
  GemmArgs p[GROUP_MAX];
};

template <int TN>
__global__ __launch_bounds__(1024 / TN) void gemm_wgrad_group_kernel(GemmGroup gg) {
  extern __shared__ __attribute__((aligned(1024))) char smem_raw[];
  const int G = gridDim.x;
  // slot of this workgroup inside a round: XCD x (workgroup ids x, x+8, ...) gets a contiguous band of the round
  const int per = G >> 3, main = per << 3;
  const int slot = (int)blockIdx.x < main ? ((int)blockIdx.x & 7) * per + ((int)blockIdx.x >> 3) : (int)blockIdx.x;
  for (int t = slot; t < gg.total_tiles; t += G) {
    int pi = 0;
    while (pi + 1 < gg.n && t >= gg.first_tile[pi + 1]) ++pi;        // wave-uniform scalar search
    const GemmArgs& g = gg.p[pi];
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    int tile_m, tile_n;
    tile_of(t - gg.first_tile[pi], tiles_m, tiles_n, tile_m, tile_n);
    gemm_tile<false, false, EPI_ACC32, TN>(g, tile_m * BM, tile_n * BN, (lds_char*)smem_raw, gg.nseg, gg.seg_delta);
  }
}

// Eight wavefronts of 128x64 or four of 128x128 per tile: the wider ones read a third less from LDS and are ahead on
// weight gradients (+2..4 %) and on input gradients with a long reduction (+7 % at K = 22016), the narrower ones on
// short reductions (an epilogue without spills, two wavefronts per SIMD to cover it); the fused SwiGLU epilogue and the
// half-height tile need the narrower ones.  Both give the same bits: every output element sums the same products in the
// same order.
constexpr int WAVE_COLS = 2, WAVE_COLS_WGRAD = 4;
constexpr int WIDE_MIN_K = 8192;       // input gradients: four wavefronts from this reduction length on

// One-time set-up (CU count, a kernel's LDS limit) sits in function-local statics, whose initialisation the language
// makes thread-safe: concurrent first calls from several threads run it once.
int cu_count() {
  static const int n_cu = [] {
    int dev = 0, n = 0;
    return (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : 256;
  }();
  return n_cu;
}

template <bool AKC, bool BKC, int EPI, int WR, int TN = WAVE_COLS>
hipError_t launch_tiles(const GemmArgs& g, hipStream_t s, int tiles_m, int tiles_n, int first, int n_wg) {
  // the ring of operand tiles; every epilogue's staging (at most 128 KiB) fits inside it
  constexpr size_t LDS = LDS_BYTES;
  auto kern = gemm_mfma_kernel<AKC, BKC, EPI, TN, WR>;
  static const hipError_t attr = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3(n_wg), dim3(WR * 512 / TN), LDS, s, g, tiles_m, tiles_n, first);
  return hipGetLastError();
}

// Full tiles for every complete round of one tile per CU; what is left over -- a last round that would keep at most
// half of the CUs busy, or a whole product with that few tiles -- goes out as twice as many half-height tiles, which
// take about two thirds as long each, or, if that would still leave half of the CUs idle and the epilogue is a plain
// one, as four times as many 128 x 128 tiles (two fifths as long each).  `shape`: 0 = this rule, 1 = full tiles only,
// 2 = half-height tiles only, 3 = 128 x 128 tiles only (where there are none: the rule).
template <bool AKC, bool BKC, int EPI>
hipError_t launch(const GemmArgs& g, hipStream_t s, int shape) {
  const int tiles_m = (g.M + BM - 1) / BM;
  const int tiles_n = EPI == EPI_SWIGLU ? (g.N / 2 + GLU_BN - 1) / GLU_BN : (g.N + BN - 1) / BN, total = tiles_m * tiles_n;
  constexpr bool QUARTERS = AKC && (EPI == EPI_STORE || EPI == EPI_RESID);
  int n_half = 0, n_quarter = 0;          // full tiles at the end of the walk order that are split in two / in four
  if constexpr (AKC) {
    const int n_cu = cu_count(), tail = total % n_cu;
    if (QUARTERS && (shape == 3 || (shape == 0 && 4 * tail <= n_cu))) n_quarter = shape == 3 ? total : tail;
    else n_half = shape == 2 ? total : shape == 1 ? 0 : (2 * tail <= n_cu ? tail : 0);
  }
  const int n_small = n_half + n_quarter;
  if (total > n_small) {
    hipError_t e;
    if constexpr (AKC && BKC && EPI == EPI_STORE)
      e = g.K >= WIDE_MIN_K ? launch_tiles<AKC, BKC, EPI, 2, 4>(g, s, tiles_m, tiles_n, 0, total - n_small)
                            : launch_tiles<AKC, BKC, EPI, 2>(g, s, tiles_m, tiles_n, 0, total - n_small);
    else
      e = launch_tiles<AKC, BKC, EPI, 2>(g, s, tiles_m, tiles_n, 0, total - n_small);
    if (e != hipSuccess) return e;
  }
  if constexpr (AKC) {
    if (n_half) return launch_tiles<AKC, BKC, EPI, 1>(g, s, tiles_m, tiles_n, total - n_half, 2 * n_half);
  }
  if constexpr (QUARTERS) {
    if (n_quarter) {
      auto kern = gemm_quarter_kernel<AKC, BKC, EPI>;
      static const hipError_t attr = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
      if (attr != hipSuccess) return attr;
      hipLaunchKernelGGL(kern, dim3(4 * n_quarter), dim3(256), LDS_BYTES, s, g, tiles_m, tiles_n, total - n_quarter);
      return hipGetLastError();
    }
  }
  return hipSuccess;
}

}  // namespace

bool gemm_mfma_supported(const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return false;
  auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  if (!al16(g.A) || !al16(g.B) || (!g.act_bwd && !al16(g.C)) || (g.R && !al16(g.R))) return false;
  if (g.lda % 8 || g.ldb % 8 || g.ldc % 4 || (g.R && g.ldr % 4) || g.N % 8) return false;
  if (!g.acc_f32 && !g.c_f32 && g.ldc % 8) return false;   // bf16 C is stored 16 bytes at a time
  const int64_t lim = (int64_t)1 << 30;   // operand byte offsets are 32-bit buffer offsets below 2 GiB
  const int64_t a_rows = g.mode == GEMM_TN ? g.K : g.M, b_rows = g.mode == GEMM_NT ? g.N : g.K;
  if (a_rows * g.lda >= lim || b_rows * g.ldb >= lim) return false;
  if (g.acc_f32 && (int64_t)g.M * g.ldc >= lim / 2) return false;   // C is read through a 32-bit byte offset too
  if (g.bias && (g.mode != GEMM_NN || ((uintptr_t)g.bias & 7))) return false;
  if (g.act_bwd) {  // fused activation backward: input-gradient product of the FFN-out map only
    if (g.mode != GEMM_NT || g.act || g.bias || g.R || g.c_f32 || g.acc_f32 || (g.act_bwd != 1 && g.act_bwd != 2) || !g.Z || !al16(g.Z) ||
        g.ldz % 8 || g.ldz < (int64_t)g.act_bwd * g.N || (int64_t)g.M * g.ldz >= lim)
      return false;
  }
  if (g.act) {     // fused activation: forward FFN-in product only
    if (g.mode != GEMM_NN || g.R || g.c_f32 || g.acc_f32 || (g.act != 1 && g.act != 2) || !g.C2 || !al16(g.C2) || g.ldc2 % 8) return false;
    if (g.act == 2 && g.N % 16) return false;      // gate | up halves of whole 16-byte pieces
  }
  switch (g.mode) {
    case GEMM_NN: return g.K % BK == 0 && !g.acc_f32;
    case GEMM_NT: return g.K % BK == 0 && !g.acc_f32 && !g.R && !g.c_f32;
    case GEMM_TN: return g.M % 8 == 0 && g.acc_f32 && !g.R && !g.c_f32;
  }
  return false;
}

hipError_t gemm_mfma(const GemmArgs& g, hipStream_t s, int tile_shape) {
  switch (g.mode) {
    case GEMM_NN:
      if (g.act == 1) return launch<true, false, EPI_GELU>(g, s, tile_shape);
      if (g.act == 2) return launch<true, false, EPI_SWIGLU>(g, s, tile_shape);
      return (g.R || g.c_f32) ? launch<true, false, EPI_RESID>(g, s, tile_shape) : launch<true, false, EPI_STORE>(g, s, tile_shape);
    case GEMM_NT:
      if (g.act_bwd == 1) return launch<true, true, EPI_DGELU>(g, s, tile_shape);
      if (g.act_bwd == 2) return launch<true, true, EPI_DSWIGLU>(g, s, tile_shape);
      return launch<true, true, EPI_STORE>(g, s, tile_shape);
    case GEMM_TN: return launch<false, false, EPI_ACC32>(g, s, tile_shape);
  }
  return hipErrorInvalidValue;
}

bool gemm_mfma_wgrad_group_supported(const GemmArgs* list, int n, int nseg, const int64_t* seg_delta) {
  if (n < 1 || nseg < 1 || nseg > GEMM_MAX_SEG || (nseg > 1 && !seg_delta)) return false;
  for (int s = 1; s < nseg; ++s)
    if (seg_delta[s] % 16) return false;
  for (int i = 0; i < n; ++i)
    if (list[i].mode != GEMM_TN || !gemm_mfma_supported(list[i])) return false;
  return true;
}

hipError_t gemm_mfma_wgrad_group(const GemmArgs* list, int n, int nseg, const int64_t* seg_delta, hipStream_t s) {
  auto kern = gemm_wgrad_group_kernel<WAVE_COLS_WGRAD>;
  static const hipError_t attr = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
  if (attr != hipSuccess) return attr;
  const int n_cu = cu_count();
  for (int i0 = 0; i0 < n; i0 += GROUP_MAX) {
    GemmGroup gg;
    gg.n = n - i0 < GROUP_MAX ? n - i0 : GROUP_MAX;
    gg.nseg = nseg;
    for (int sg = 0; sg < GEMM_MAX_SEG; ++sg) gg.seg_delta[sg] = (sg > 0 && sg < nseg) ? seg_delta[sg] : 0;
    int total = 0;
    for (int i = 0; i < gg.n; ++i) {
      gg.p[i] = list[i0 + i];
      gg.first_tile[i] = total;
      total += ((gg.p[i].M + BM - 1) / BM) * ((gg.p[i].N + BN - 1) / BN);
    }
    for (int i = gg.n; i <= GROUP_MAX; ++i) gg.first_tile[i] = total;
    gg.total_tiles = total;
    const int grid = total < n_cu ? total : n_cu;       // one workgroup per CU (128 KiB of LDS each)
    hipLaunchKernelGGL(kern, dim3(grid), dim3(1024 / WAVE_COLS_WGRAD), LDS_BYTES, s, gg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace stg
