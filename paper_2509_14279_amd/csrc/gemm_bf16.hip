// bf16 MFMA GEMM for the three contractions of the fused dense-layer block (gfx950).
//
//     D[i][j] = sum_r P(i,r) * Q(j,r)      stored as C[j][i]   (C row-major, leading dimension I)
//
// P feeds the MFMA "A" side, Q the "B" side, so a lane ends up with 4 consecutive i (output columns) of one
// output row j in adjacent accumulator registers, and a row reduction over i (the LayerNorm statistics, where
// the forward pass takes them here) is a sum inside the lane plus one cross-half exchange.
//
//   F1  Z[m][n]  = sum_k X[m][k] W[n][k] + b[n]   P = W (i = n, r-contiguous)   Q = X  (j = m, r-contiguous)
//       or, for large batches,                    P = W^T (a transposed copy: r = k major)
//       (also the forward product of the sibling operators: Linear+ReLU, its backward pass's recomputation of the
//        pre-activation with the activation mask applied to the upstream gradient, and the three products of the
//        gated feed-forward block)
//   B3  dX[m][k] = sum_n dZ[m][n] W[n][k]         P = W (i = k, r = n major)    Q = dZ (j = m, r-contiguous)
//   B4  dW[n][k] = sum_m dZ[m][n] X[m][k]         P = X (i = k, r = m major)    Q = dZ (j = n, r = m major)
//       (dZ is the library's own buffer and may be stored in 32 x 32 blocks, which suits both of its readers: Loader)
// (the linear layer's forward, grad-input and grad-weight products of the paper's linear tasks.)
//
// Workgroup: 256 threads = 4 waves (2 x 2), one per SIMD; block tile 256 x 256, wave tile 128 x 128 as 4 x 4
// v_mfma_f32_32x32x16_bf16 blocks (256 fp32 accumulators per lane, held in AGPRs).  The reduction runs in slices of
// BK through NS LDS stages (BK x NS = 64 x 2 or 32 x 4, 128 KB either way) filled by direct global->LDS loads
// (16 bytes per lane, no staging registers); the loads of slice kt+NS are issued as soon as slice kt's stage is
// released and stay in flight for NS-1 slice times while the MFMAs of the other stages run.  Workgroups are
// persistent (one per CU): the first slices of a workgroup's next tile are fetched during the last slices of its
// current one, and output tiles leave through a small LDS staging area as 256-byte row segments (short row
// segments cost write bandwidth: 8 or 16 bytes per lane straight from the registers measured 3 to 18 % slower).
// The number of slices per tile is a multiple of NS, so every slice's LDS stage is a compile-time constant.
//
// LDS tile layouts (XOR-swizzled by choosing which global chunk a lane fetches, since a direct load lands at
// base + lane*16).  The LDS of this part has 64 banks of 4 bytes; a 16-byte read serves the wavefront in four groups
// of 16 lanes - lanes {0-3, 12-15, 20-23, 24-27}, {4-11, 16-19, 28-31} and the same plus 32, measured with a pairwise
// conflict probe - and an 8-byte read in two groups of 32 consecutive lanes; a group completes in one cycle when
// its lanes touch 64 distinct banks.
//   r-contiguous operand: [256 rows][BK/8 chunks of 16 B]; BK = 64 (rows of 128 B, two rows per bank round): chunk c
//       of row w in slot c ^ ((w >> 1) & 7); BK = 32 (rows of 64 B, four rows per bank round): slot c ^ ((w >> 2) & 3);
//       fragments are read with ds_read_b128 (8 consecutive r of the lane's row): the 16 rows of a lane group then
//       cover all 64 banks.
//   r-major operand:      [BK r-rows][32 chunks of 16 B]; chunk c of r-row w sits in slot c ^ ((w & 3) << 2);
//       fragments are read with the transposing ds_read_b64_tr_b16 (4 consecutive r for the lane's column): the 32
//       lanes of a group read 64 bytes from each of 4 r-rows, which the swizzle spreads over the 256-byte bank round.
#include "common.hip.h"
#include "internal.h"

#include <type_traits>

namespace fdl {
namespace {

constexpr int kTile = 256;
// The launch plan (workspace sizes included) is host-only and must not depend on which device runs it, so the split
// of the dW reduction is planned for the part's 256 compute units; the launch itself asks the device.
constexpr int kPlanCUs = 256;
constexpr int kLdsStages = 128 * 1024;           // all pipeline stages together (2 x 64 KB or 4 x 32 KB)
constexpr int kLdsBytes = kLdsStages + 4 * 8192; // + 8 KB per wave for the output block rows = 160 KB

// Geometry of one pipeline configuration: reduction slices of BK, NS stages.
template <int BK> struct Geo {
  static constexpr int kSub = BK / 16;                    // MFMA sub-slices per slice
  static constexpr int kOperandBytes = kTile * BK * 2;    // one operand tile of one slice
  static constexpr int kStageBytes = 2 * kOperandBytes;   // P tile then Q tile
  static constexpr int kDpw = BK / 8;                     // direct-load instructions per operand, wave and slice
  static constexpr int kWaveBytes = kOperandBytes / 4;    // each wave fills a quarter of an operand tile
};

// EPI_STORE: C = acc.  EPI_BIAS: C = acc + bias.  EPI_F1: EPI_BIAS plus GELU and partial row statistics.
// EPI_PARTIAL: fp32 partial sums of a split reduction.  EPI_RELU: C = max(acc + bias, 0).
// EPI_MASK: C = aux where acc + bias > 0, else 0 (aux [J][I]: the upstream gradient of a ReLU).
// EPI_GATE: two P operands (gate and up weights), C = SiLU(Q P^T) * (Q P2^T): see the kernel's p_origin.
enum { EPI_STORE = 0, EPI_F1 = 1, EPI_BIAS = 2, EPI_PARTIAL = 3, EPI_RELU = 4, EPI_MASK = 5, EPI_GATE = 6 };

struct FastParams {
  const bf16_t* P; const bf16_t* Q;
  const bf16_t* P2;      // EPI_GATE: the second P operand (same shape and pitch as P)
  const bf16_t* Qtail;   // RAG: the Q rows of the last (partial) row tile as a padded 256-row copy, or null if Q
                         //      itself has readable rows up to the end of that tile
  int64_t ldp, ldq;
  bf16_t* C;             // [J][I]
  float* Cpart;          // [split][J][I] fp32 (split > 1)
  const float* bias;     // [I]   (EPI_F1, EPI_BIAS, EPI_RELU, EPI_MASK)
  const bf16_t* aux;     // [J][I] (EPI_MASK)
  f32x2* part;           // [I/128][J]  (EPI_F1)
  int I, J;              // J: valid output rows (RAG: any number >= 1; otherwise a multiple of 256)
  int tiles_i, tiles_j;
  int nkt;               // reduction slices per workgroup
  int split;
  int xcds;              // accelerator dies the workgroup ids are dealt over (1: no die-aware tile order)
  int qblocked;          // 1: Q (the library's own dZ buffer, ldq columns) is stored in blocks of 32 x 32, see Loader
  int cblocked;          // 1: the output C [J][I] is written in that blocked layout (EPI_MASK: the masked gradient;
                         //    EPI_GATE: the gated activation)
};

typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((ext_vector_type(4))) short short4_;
typedef __attribute__((address_space(3))) short4_ lds_short4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;

// 16 bytes per lane, global -> LDS, no registers: lane l's data lands at (lds_base + LDS_OFF) + 16 l.
// voff: per-lane byte offset, sbase: wave-uniform global base, lds_base: wave-uniform LDS byte address.
// M0 carries the LDS address; one wait state separates the SALU write of M0 from the load that reads it.
template <int LDS_OFF>
__device__ __forceinline__ void dma16(uint32_t voff, const void* sbase, uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(sbase), "s"(lds_base), "n"(LDS_OFF) : "memory", "m0", "scc");
}
// 4 bytes per lane: lane l's dword lands at (lds_base + LDS_OFF) + 4 l
template <int LDS_OFF>
__device__ __forceinline__ void dma4(uint32_t voff, const void* sbase, uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :: "v"(voff), "s"(sbase), "s"(lds_base), "n"(LDS_OFF) : "memory", "m0", "scc");
}
// wait until at most N vector-memory operations of this wave are outstanding (loads complete in order)
template <int N> __device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

template <bool RM, int BK> struct Loader {
  // voff[q]: per-lane byte offset of instruction q (constant over the reduction loop).  kDpw instructions per wave
  // fill this wave's quarter of the operand tile; the only per-slice scalar work is one base pointer.
  // Blocked operand (BK = 32 only): the matrix [rows][ld] is stored as [rows / 32][ld / 32] blocks of 32 x 32
  // elements, each block row-major and 2 KB long.  Either orientation then reads long runs: a 256-row slice of 32
  // reduction columns (r-contiguous use) is 8 whole blocks, a slice of 32 reduction rows by 256 columns (r-major use)
  // is 8 neighbouring blocks, 16 KB in one piece - where a row-major matrix gives the r-contiguous reader 256 runs of
  // 64 bytes, half a cache line each, whose other half it asks for again one slice later.  The 16-byte chunk a lane
  // fetches and the LDS slot it lands in are the same as for a row-major operand; only its address differs.
  static constexpr int kDpw = Geo<BK>::kDpw;
  uint32_t voff[kDpw];
  int blocked;
  __device__ __forceinline__ void init(int lane, int64_t ld, int blocked_operand = 0) {
    blocked = (BK == 32) ? blocked_operand : 0;
#pragma unroll
    for (int q = 0; q < kDpw; q++) {
      if (BK == 32 && blocked && RM) {
        // r-row 2q + h of this wave's 8 (all in one block row), chunk c: block c / 4, 16-byte piece c % 4 of its row
        const int h = lane >> 5, slot = lane & 31;
        const int c = slot ^ (((2 * q + h) & 3) << 2);
        voff[q] = (uint32_t)((c >> 2) * 2048 + (2 * q + h) * 64 + (c & 3) * 16);
      } else if (BK == 32 && blocked) {
        // row 16q + w of this wave's 64 (two block rows), piece slot ^ swizzle of its 64 bytes in the block
        const int w = lane >> 2, slot = lane & 3, rr = 16 * q + w;
        voff[q] = (uint32_t)((int64_t)(rr >> 5) * (ld >> 5) * 2048 + (rr & 31) * 64 + ((slot ^ ((w >> 2) & 3)) * 16));
      } else if (RM) {
        // instruction q covers r-rows 2q, 2q+1 of this wave's BK/4; lane: r-row 2q + h, h = lane/32, slot lane%32
        const int h = lane >> 5, slot = lane & 31;
        const int c = slot ^ (((2 * q + h) & 3) << 2);
        voff[q] = (uint32_t)((int64_t)(2 * q + h) * ld * 2 + c * 16);
      } else if (BK == 64) {
        // instruction q covers rows 8q..8q+7 of this wave's 64; lane: row 8q + w, w = lane/8, slot lane%8
        const int w = lane >> 3, slot = lane & 7;
        voff[q] = (uint32_t)((int64_t)(8 * q + w) * ld * 2 + ((slot ^ ((4 * q + (w >> 1)) & 7)) * 16));
      } else {
        // BK = 32: instruction q covers rows 16q..16q+15 of this wave's 64; lane: row 16q + w, w = lane/4, slot lane%4
        const int w = lane >> 2, slot = lane & 3;
        voff[q] = (uint32_t)((int64_t)(16 * q + w) * ld * 2 + ((slot ^ ((w >> 2) & 3)) * 16));
      }
    }
  }
  // first element this wave fetches of the slice that starts at `base` (block tile origin, first r of the slice)
  __device__ __forceinline__ const bf16_t* wave_base(const bf16_t* base, int64_t ld, int wave) const {
    if (BK == 32 && blocked) return RM ? base + wave * (BK / 4) * 32 : base + (int64_t)(wave * 2) * (ld >> 5) * 1024;
    return RM ? base + (int64_t)(wave * (BK / 4)) * ld : base + (int64_t)(wave * 64) * ld;
  }
  // wbase: wave_base(...) of the slice; wlds: LDS address of this wave's quarter of the operand tile
  template <int Q> __device__ __forceinline__ void issue1(const bf16_t* wbase, uint32_t wlds) const {
    dma16<Q * 1024>(voff[Q < kDpw ? Q : 0], wbase, wlds);
  }
  // q is a compile-time constant at every call site once the surrounding loop is unrolled
  __device__ __forceinline__ void issue_q(int q, const bf16_t* wbase, uint32_t wlds) const {
    switch (q) {
      case 0: issue1<0>(wbase, wlds); break;
      case 1: issue1<1>(wbase, wlds); break;
      case 2: issue1<2>(wbase, wlds); break;
      case 3: issue1<3>(wbase, wlds); break;
      case 4: if (kDpw > 4) issue1<4>(wbase, wlds); break;
      case 5: if (kDpw > 4) issue1<5>(wbase, wlds); break;
      case 6: if (kDpw > 4) issue1<6>(wbase, wlds); break;
      default: if (kDpw > 4) issue1<7>(wbase, wlds); break;
    }
  }
  __device__ __forceinline__ void issue(const bf16_t* wbase, uint32_t wlds) const {
#pragma unroll
    for (int q = 0; q < kDpw; q++) issue_q(q, wbase, wlds);
  }
};

template <bool RM, int BK> struct Frags {
  // LDS byte offsets of this lane's fragment reads inside an operand tile.
  //  r-contiguous: off[kk] for the sub-slices; block a adds a * 32 rows.
  //  r-major:      off[a] for the 4 blocks; sub-slice kk and half t add (kk*16 + 4t)*512.
  uint32_t off[4];
  __device__ __forceinline__ void init(int lane, int w /* wave coordinate along this operand */) {
    if (RM) {
      const int G = lane >> 4, p = lane & 15;
      const int r = 8 * (G >> 1) + (p >> 2);
#pragma unroll
      for (int a = 0; a < 4; a++) {
        const int c = w * 16 + a * 4 + 2 * (G & 1) + ((p & 3) >> 1);
        off[a] = (uint32_t)(r * 512 + ((c ^ ((p >> 2) << 2)) * 16) + (p & 1) * 8);
      }
    } else if (BK == 64) {
      // rows of 128 B, chunk c of row r in slot c ^ ((r >> 1) & 7)
      const int row = w * 128 + (lane & 31);
      const int t0 = (lane >> 5) ^ ((lane >> 1) & 7);
#pragma unroll
      for (int kk = 0; kk < 4; kk++) off[kk] = (uint32_t)(row * 128 + (((kk << 1) ^ t0) << 4));
    } else {
      // rows of 64 B, chunk c of row r in slot c ^ ((r >> 2) & 3)
      const int row = w * 128 + (lane & 31);
      const int sw = (lane >> 2) & 3;
#pragma unroll
      for (int kk = 0; kk < 4; kk++) off[kk] = (uint32_t)(row * 64 + (((((kk & 1) << 1) | (lane >> 5)) ^ sw) << 4));
    }
  }
  __device__ __forceinline__ bf16x8 load(const lds_char* tile, int a, int kk) const {
    if (RM) {
      const lds_char* p0 = tile + off[a] + (kk * 16) * 512;
      const short4_ lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)p0);
      const short4_ hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4*)(p0 + 4 * 512));
      typedef __attribute__((ext_vector_type(8))) short short8_;
      short8_ v;
      v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3]; v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
      return __builtin_bit_cast(bf16x8, v);
    } else {
      typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
      return *(const lds_bf16x8*)(tile + off[kk] + a * (32 * BK * 2));
    }
  }
};

// Output tile of a logical tile index: bands of 8 output-row tiles, walked column-tile-major inside a band.
struct TileCoord { int i0, j0; };
__device__ __forceinline__ TileCoord tile_coord(int L, int tiles_i, int tiles_j) {
  const int band_tiles = 8 * tiles_i;
  const int band = L / band_tiles;
  const int rem = L - band * band_tiles;
  int band_h = tiles_j - band * 8;
  if (band_h > 8) band_h = 8;
  TileCoord c;
  c.i0 = (rem / band_h) * kTile;
  c.j0 = (band * 8 + rem % band_h) * kTile;
  return c;
}

// RAG: the number of output rows J is not a multiple of the tile (ragged batch dimension of F1 and B3, ragged N of
// B4).  The last row tile then reads its Q rows from a padded copy (or from a Q buffer that is itself padded), computes
// the surplus rows on whatever that padding holds - rows of a product are independent - and does not store them.
// CRAG (with RAG): the number of output columns I is a multiple of 8 but not of the tile.  The host hands over a P
// operand that is readable up to the end of the last column tile (a zero-padded copy of the weights, or a matrix
// whose surplus columns are the start of its next row) and a bias padded likewise; the surplus columns are computed
// and not stored, and are left out of the row statistics where the epilogue takes them.
// A reduction length that is not a whole number of pipeline rounds is the host's business as well: it rounds the
// length up and makes one operand zero over the surplus (the other only has to be readable and finite there).
// The body of the kernel: the persistent tile loop of workgroup `bid` of `nblk` on reduction part `part`.  It is a
// function of its own so that one launch can carry two contractions side by side (see gemm_bf16_pair_kernel).
template <bool P_RM, bool Q_RM, int EPI, int BK, int NS, bool RAG, bool CRAG = false>
__device__ __forceinline__ void gemm_tile_loop(const FastParams& p, char* smem, const int bid, const int nblk, const int part) {
  static_assert(!CRAG || RAG, "ragged columns come with the ragged-row checks");
  typedef Geo<BK> G;
  static_assert(NS * G::kStageBytes == kLdsStages, "stages must fill 128 KB");
  static_assert((NS == 2 || NS == 4) && (G::kSub & 1) == 0, "2 or 4 stages, even number of sub-slices");
  lds_char* lds = (lds_char*)smem;
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wi = wave & 1, wj = wave >> 1;

  // ---- persistent workgroups: one per CU, each walks several output tiles.  Workgroup ids are dealt round-robin
  // over the X accelerator dies (8 on this part), so die x owns the logical tiles [x T/X, (x+1) T/X) and its
  // workgroups take them in turn: the 32 workgroups resident on a die work on 32 consecutive logical tiles (4 column
  // tiles x 8 row tiles of one band) and share 4 P panels and 8 Q panels in that die's L2.  The host passes X > 1
  // only when both the tile count and the grid are multiples of it.
  const int ntiles = p.tiles_i * p.tiles_j;
  int L, Lstride, Lend;
  if (p.xcds > 1) {
    const int X = p.xcds;
    const int per_xcd = ntiles / X;
    const int xcd = bid % X, slot = bid / X;
    L = xcd * per_xcd + slot;
    Lstride = nblk / X;
    Lend = (xcd + 1) * per_xcd;
  } else {
    L = bid; Lstride = nblk; Lend = ntiles;
  }
  const int64_t r_begin = (int64_t)part * p.nkt * BK;

  // Per-lane offsets of the direct loads and of the fragment reads.  They are recomputed at the top of every tile
  // (from a copy of the lane id the compiler cannot see through) rather than kept across the epilogue, where the
  // register allocator would otherwise park them in scratch memory: a reload there has to wait for every output
  // store issued before it, because vector memory operations retire in order.
  Loader<P_RM, BK> lp; Loader<Q_RM, BK> lq;
  Frags<P_RM, BK> fp; Frags<Q_RM, BK> fq;
  auto init_offsets = [&]() {
    int lt = lane;
    asm volatile("" : "+v"(lt));
    lp.init(lt, p.ldp); lq.init(lt, p.ldq, p.qblocked);
    fp.init(lt, wi); fq.init(lt, wj);
  };
  init_offsets();   // for the initial fill below; every tile recomputes them

  const int64_t pstep = P_RM ? (int64_t)BK * p.ldp : BK;
  const bool qblk = BK == 32 && p.qblocked != 0;
  // (a slice step of an r-major operand is 32 rows = one block row either way: 32 ldq elements)
  const int64_t qstep = Q_RM ? (int64_t)BK * p.ldq : (qblk ? 1024 : BK);
  // first element this wave fetches of slice 0 of the tile at (i0, j0)
  // EPI_GATE: the 256 rows of a P tile are 64 gate rows, the same 64 up rows, the next 64 gate rows and their up rows
  // (rows of P and P2 from i0/2 on), one quarter per wave: a wave's accumulator blocks a = 0, 1 then hold the gate
  // product and a = 2, 3 the up product of the same 64 output columns, register for register, and the gated
  // activation needs no exchange between lanes.  The tile is 128 output columns wide.
  auto p_origin = [&](int i0) {
    if (EPI == EPI_GATE && !P_RM)   // (an r-major P for this epilogue is one matrix with that row order built in)
      return ((wave & 1) ? p.P2 : p.P) + (int64_t)((i0 >> 1) + (wave >> 1) * 64) * p.ldp + r_begin;
    return lp.wave_base(P_RM ? p.P + r_begin * p.ldp + i0 : p.P + (int64_t)i0 * p.ldp + r_begin, p.ldp, wave);
  };
  auto q_origin = [&](int j0) {
    if (RAG && !Q_RM && p.Qtail != nullptr && j0 == (p.tiles_j - 1) * kTile) return lq.wave_base(p.Qtail + r_begin, p.ldq, wave);
    if (qblk)   // block (j0 / 32, r_begin / 32), or (r_begin / 32, j0 / 32) for the r-major reader
      return lq.wave_base(Q_RM ? p.Q + ((r_begin >> 5) * (p.ldq >> 5) + (j0 >> 5)) * 1024
                               : p.Q + ((int64_t)(j0 >> 5) * (p.ldq >> 5) + (r_begin >> 5)) * 1024, p.ldq, wave);
    return lq.wave_base(Q_RM ? p.Q + r_begin * p.ldq + j0 : p.Q + (int64_t)j0 * p.ldq + r_begin, p.ldq, wave);
  };

  const int nkt = p.nkt;                                                  // >= NS
  const uint32_t wlds = lds0 + (uint32_t)wave * (uint32_t)G::kWaveBytes;  // this wave's quarter of an operand tile
  TileCoord tc = tile_coord(L, p.tiles_i, p.tiles_j);
  const bf16_t* pcur = p_origin(tc.i0);
  const bf16_t* qcur = q_origin(tc.j0);
#pragma unroll
  for (int st = 0; st < NS; st++) {
    lp.issue(pcur + st * pstep, wlds + st * G::kStageBytes);
    lq.issue(qcur + st * qstep, wlds + st * G::kStageBytes + G::kOperandBytes);
  }
  // the slice fetched last, as (addresses, index inside its tile)
  const bf16_t* pfetch = pcur + (NS - 1) * pstep;
  const bf16_t* qfetch = qcur + (NS - 1) * qstep;
  int fidx = NS - 1;
  wait_dma<0>();
  __syncthreads();

  // Fragments are double-buffered in registers: while the 16 MFMAs of a sub-slice run, the 8 fragment reads of the
  // next sub-slice are issued between them.  The last sub-slice's MFMAs are issued after the barrier that
  // publishes the next stage, behind the first fragment reads of that stage, so the matrix pipe has work while
  // those reads are in flight.
  bf16x8 pf[2][4], qf[2][4];

  const int half = lane >> 5, l32 = lane & 31;
  typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

  // Forward: the bias enters through the matrix pipe as one extra reduction step after the last slice,
  // acc += Pb Qb^T with Pb[i][0..2] = the three bf16 pieces of bias[i] (hi + mid + lo = the fp32 value exactly:
  // 3 x 8 significant bits) and Qb[j][0..2] = 1: sixteen MFMAs per tile and no vector arithmetic in the epilogue.
  // A lane needs the bias of one column per block a (only lanes 0..31 carry k = 0..7).  The wave's 128 bias
  // values are fetched at the top of the tile by two direct loads into its output staging area, which is idle
  // until the epilogue: like every direct load they are older than the slice loads issued after them, so the main
  // loop's own waits cover them, and no register or compiler-inserted wait is involved.
  constexpr bool kBias = EPI == EPI_BIAS || EPI == EPI_F1 || EPI == EPI_RELU || EPI == EPI_MASK;

  for (;;) {
    // slice 0 of this tile has landed in stage 0 (initial fill, or prefetched during the previous tile and
    // published by its last barrier): first fragments
    init_offsets();
#pragma unroll
    for (int a = 0; a < 4; a++) pf[0][a] = fp.load(lds, a, 0);
#pragma unroll
    for (int b = 0; b < 4; b++) qf[0][b] = fq.load(lds + G::kOperandBytes, b, 0);

    // the tile after this one (its first NS slices are fetched during this tile's last NS slices); a workgroup
    // without a next tile fetches its own last slice again instead (never read)
    const int Ln = L + Lstride;
    const bool has_next = Ln < Lend;
    const TileCoord tn = tile_coord(has_next ? Ln : L, p.tiles_i, p.tiles_j);
    // where the fetch stream continues after this tile's last slice
    const bf16_t* pwrap = has_next ? p_origin(tn.i0) : p_origin(tc.i0) + (int64_t)(nkt - 1) * pstep;
    const bf16_t* qwrap = has_next ? q_origin(tn.j0) : q_origin(tc.j0) + (int64_t)(nkt - 1) * qstep;
    const int fwrap = has_next ? 0 : nkt - 1;

    if (kBias) {
      int lb = lane;
      asm volatile("" : "+v"(lb));
      const float* bsrc = p.bias + tc.i0 + wi * 128;
      const uint32_t wst = lds0 + (uint32_t)kLdsStages + (uint32_t)wave * 8192u;
      dma4<0>((uint32_t)lb * 4u, bsrc, wst);
      dma4<256>((uint32_t)lb * 4u, bsrc + 64, wst);
    }

    // The accumulators are never cleared: the first sub-slice of a tile's slice 0 runs its MFMAs with a zero
    // addend (slice 0 has its own copy of the slice code for that; the other slices, at least NS-1 of them -
    // checked on the host - run in the loop).
    f32x16 acc[4][4];
    f32x16 zero16;
#pragma unroll
    for (int r = 0; r < 16; r++) zero16[r] = 0.0f;

    // One slice; the LDS stage it lives in is a compile-time constant (the number of slices per tile is a multiple
    // of NS - checked on the host - so a tile's slice 0 is always in stage 0 and the slice loop is unrolled NS
    // times): every LDS address is then a per-lane register plus an immediate.
    auto slice = [&](auto stage_tag, auto first_tag) {
      constexpr bool kFirst = decltype(first_tag)::value;
      constexpr int cur = decltype(stage_tag)::value;
      constexpr int nxt = (cur + 1) & (NS - 1);
      // Slice kt+NS is fetched into this slice's own stage as soon as the barrier below has shown that every wave
      // holds its last fragments of slice kt in registers; those direct loads then have NS-1 slice times before
      // the barrier that publishes them.  (pfetch, qfetch, fidx) name the slice fetched last and are stepped in
      // the shadow of the last sub-slice's first MFMA: a handful of scalar instructions, where recomputing the
      // addresses from the slice index cost two dozen in front of every slice's first MFMA.
      const uint32_t own = wlds + (uint32_t)cur * G::kStageBytes;
      const lds_char* tp = lds + cur * G::kStageBytes;
      const lds_char* tq = tp + G::kOperandBytes;
      const lds_char* np_ = lds + nxt * G::kStageBytes;
      const lds_char* nq_ = np_ + G::kOperandBytes;
      // Issue order is pinned by hand (a scheduling barrier after every step): MFMA t of a sub-slice is followed
      // by a fragment read of the next sub-slice (even t) and, in the last sub-slice, by a direct load, so
      // neither the LDS reads nor the global loads keep the matrix pipe waiting for long.
#pragma unroll
      for (int kk = 0; kk < G::kSub; kk++) {
        const int use = kk & 1, fill = use ^ 1;
        const bool lastsub = kk == G::kSub - 1;
        if (lastsub) {
          // slice kt+1 must have landed; the direct loads of the NS-2 slices after it may stay in flight
          wait_dma<(NS - 2) * 2 * G::kDpw>();
          __syncthreads();
          __builtin_amdgcn_sched_barrier(0);
        }
        const lds_char* rp = lastsub ? np_ : tp;
        const lds_char* rq = lastsub ? nq_ : tq;
        const int rk = lastsub ? 0 : kk + 1;
#pragma unroll
        for (int t = 0; t < 16; t++) {
          const int a = t >> 2, b = t & 3;
          if (kFirst && kk == 0)
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[use][a], qf[use][b], zero16, 0, 0, 0);
          else
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[use][a], qf[use][b], acc[a][b], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          // next slice of the fetch stream: the following one of this tile, else (pwrap, qwrap, fwrap) = slice 0
          // of the next tile or, without a next tile, this tile's last slice again, which is never read; spread
          // over three MFMA shadows
          if (lastsub && t == 0) {
            pfetch = fidx + 1 == nkt ? pwrap : pfetch + pstep;
            __builtin_amdgcn_sched_barrier(0);
          }
          if (lastsub && t == 2) {
            qfetch = fidx + 1 == nkt ? qwrap : qfetch + qstep;
            __builtin_amdgcn_sched_barrier(0);
          }
          if (lastsub && t == 4) {
            fidx = fidx + 1 == nkt ? fwrap : fidx + 1;
            __builtin_amdgcn_sched_barrier(0);
          }
          const bf16_t* const pn = pfetch;
          const bf16_t* const qn = qfetch;
          if ((t & 1) == 0) {
            // read order: P0, Q0, Q1, Q2, Q3, P1, P2, P3 (the order in which the next sub-slice consumes them)
            const int slot = t >> 1;
            if (slot == 0) pf[fill][0] = fp.load(rp, 0, rk);
            else if (slot <= 4) qf[fill][slot - 1] = fq.load(rq, slot - 1, rk);
            else pf[fill][slot - 4] = fp.load(rp, slot - 4, rk);
            __builtin_amdgcn_sched_barrier(0);
          }
          if (lastsub) {
            if (G::kDpw == 8) {            // 16 direct loads: one behind every MFMA
              if (t < 8) lp.issue_q(t, pn, own);
              else lq.issue_q(t - 8, qn, own + G::kOperandBytes);
              __builtin_amdgcn_sched_barrier(0);
            } else if (t & 1) {            // 8 direct loads: one behind every other MFMA
              const int d = t >> 1;
              if (d < 4) lp.issue_q(d, pn, own);
              else lq.issue_q(d - 4, qn, own + G::kOperandBytes);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
      }
    };
    auto group = [&](auto first_tag) {
      slice(std::integral_constant<int, 0>(), first_tag);
      slice(std::integral_constant<int, 1>(), std::false_type());
      if constexpr (NS == 4) {
        slice(std::integral_constant<int, 2>(), std::false_type());
        slice(std::integral_constant<int, 3>(), std::false_type());
      }
    };
    group(std::true_type());
    for (int g = NS; g < nkt; g += NS) group(std::false_type());
    // here: the next tile's slice 0 has landed in stage 0, its following slices are in flight

    // ---------------------------------------------------------------- epilogue of tile (tc.i0, tc.j0)
    // Accumulator register r of block (a, b): i = a*32 + (r/4)*8 + (lane/32)*4 + r%4, j = b*32 + lane%32.  A lane's
    // four adjacent values are only 8 bytes of an output row, so bf16 tiles leave through LDS: each wave owns 8 KB
    // beyond the pipeline stages, writes one block row (32 output rows x 256 B) as [32 rows][32 units of 8 B] with
    // unit u of row w in slot u ^ ((w & 15) << 1) (conflict-free both ways), reads it back 16 bytes per lane and
    // stores 256 contiguous bytes per row.
    // Every per-lane constant of the epilogue is derived here from a copy of the lane id the compiler cannot see
    // through: hoisted out of the tile loop they would be spilled around the main loop, and each reload in the
    // epilogue would wait for the output stores issued before it (vector memory operations retire in order).
    if (kBias) {
      bf16x8 ones, bfrag[4];
#pragma unroll
      for (int e = 0; e < 8; e++) ones[e] = (bf16_t)(e < 3 ? 1.0f : 0.0f);
#pragma unroll
      for (int a = 0; a < 4; a++) {
        typedef __attribute__((address_space(3))) float lds_float;
        const float xb = *(const lds_float*)(lds + kLdsStages + wave * 8192 + (a * 32 + l32) * 4);
        const float x = half == 0 ? xb : 0.0f;
        const bf16_t hi = (bf16_t)x;
        const float r1 = x - (float)hi;
        const bf16_t mid = (bf16_t)r1;
        const bf16_t lo = (bf16_t)(r1 - (float)mid);
#pragma unroll
        for (int e = 0; e < 8; e++) bfrag[a][e] = (bf16_t)0.0f;
        bfrag[a][0] = hi; bfrag[a][1] = mid; bfrag[a][2] = lo;
      }
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfrag[a], ones, acc[a][b], 0, 0, 0);
    }
    if (!kBias) {
      // give the register allocator a fresh start for the accumulators here, as the bias MFMAs do in the forward
      // kernels (without it, it parks a few of them in scratch memory across the epilogue)
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int b = 0; b < 4; b++) asm volatile("" : "+a"(acc[a][b]));
    }
    int le = lane;
    asm volatile("" : "+v"(le));
    const int e_half = le >> 5, e_l32 = le & 31;
    const int i0 = tc.i0, j0 = tc.j0;
    const int jw = j0 + wj * 128 + e_l32;          // + b*32
    lds_char* wtile = lds + kLdsStages + wave * 8192;
    uint32_t woff[4][4];                         // LDS byte offset of the lane's 8-byte unit (a, g) in row lane%32
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int g = 0; g < 4; g++)
        woff[a][g] = (uint32_t)(e_l32 * 256 + (((a * 8 + g * 2) ^ ((e_l32 & 15) << 1)) + e_half) * 8);
    // read side: rows it*4 + lane/16 of the block row, 16-byte chunk lane%16 (slot chunk ^ (row & 15))
    const int e_m = le & 15, e_rq = le >> 4;
    uint32_t roff[4];
#pragma unroll
    for (int c = 0; c < 4; c++) roff[c] = (uint32_t)((c * 4 + e_rq) * 256 + ((e_m ^ (c * 4 + e_rq)) << 4));
    const uint32_t svoff = (uint32_t)(e_rq * p.I + e_m * 8) * 2u;   // byte offset of the lane inside 4 output rows
    // Block row b of the wave tile (32 output rows) leaves as soon as it is complete.
    auto flush_rows = [&](int b) {
      // wave-uniform base of row it*4 of the block row; the lane adds (lane/16) rows and 16 (lane%16) bytes
      char* cbase = reinterpret_cast<char*>(p.C + (int64_t)(j0 + wj * 128 + b * 32) * p.I + i0 + wi * 128);
#pragma unroll
      for (int it = 0; it < 8; it++) {
        const u32x4 v = *(const lds_u32x4*)(wtile + roff[it & 3] + (it >> 2) * 4096);
        u32x4* dst = reinterpret_cast<u32x4*>(cbase + (int64_t)(it * 4) * p.I * 2 + svoff);
        if (EPI == EPI_MASK && p.cblocked) {
          // row R0 + lane/16 (R0 a multiple of 4, so the four rows share a block row), columns col .. col + 7:
          // four rows x 64 bytes of each of the four blocks = 256 contiguous bytes per block
          const int64_t R0 = j0 + wj * 128 + b * 32 + it * 4;
          const int col = i0 + wi * 128 + e_m * 8;
          dst = reinterpret_cast<u32x4*>(p.C + (((R0 >> 5) * (p.I >> 5) + (col >> 5)) << 10) + (((R0 & 31) + e_rq) << 5) + (col & 31));
        }
        if (RAG && j0 + wj * 128 + b * 32 + it * 4 + e_rq >= p.J) continue;   // a row past the end
        if (CRAG && i0 + wi * 128 + e_m * 8 >= p.I) continue;                  // 8 columns past the end
        if (EPI == EPI_MASK) {
          // v: 8 pre-activations as bf16.  The upstream gradient passes where the pre-activation is positive (bits
          // 0x0001 .. 0x7fff: sign clear, magnitude non-zero) and is zero elsewhere.
          const char* abase = reinterpret_cast<const char*>(p.aux + (int64_t)(j0 + wj * 128 + b * 32) * p.I + i0 + wi * 128);
          const u32x4 d = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(abase + (int64_t)(it * 4) * p.I * 2 + svoff));
          u32x4 g;
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const uint32_t lo = ((v[e] & 0xffffu) - 1u) < 0x7fffu ? 0x0000ffffu : 0u;
            const uint32_t hi = ((v[e] >> 16) - 1u) < 0x7fffu ? 0xffff0000u : 0u;
            g[e] = d[e] & (lo | hi);
          }
          *dst = g;
          continue;
        }
        // the forward output (Zsave, far larger than the caches) is streamed past them so that it does not evict
        // the operand panels the XCD's workgroups share; the smaller gradient outputs gain nothing from that
        if (kBias && EPI != EPI_MASK) __builtin_nontemporal_store(v, dst);
        else *dst = v;
      }
    };
    if (EPI == EPI_GATE) {
      // H = SiLU(gate) * up for this wave's 64 columns x 128 rows, one block row of 32 rows at a time through the
      // staging area (units 0..15 of each 256-byte staging row), stored as 128-byte row segments
      const int h0 = (i0 >> 1) + wi * 64;
      const int g_m = le & 7, g_rq = le >> 3;      // read side: 16-byte chunk lane%8 of row it*8 + lane/8
#pragma unroll
      for (int b = 0; b < 4; b++) {
#pragma unroll
        for (int a = 0; a < 2; a++)
#pragma unroll
          for (int g = 0; g < 4; g++) {
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const float z = acc[a][b][g * 4 + e], u = acc[a + 2][b][g * 4 + e];
              const float sg = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * z));
              v[e] = (bf16_t)(z * sg * u);
            }
            *(lds_bf16x4*)(wtile + woff[a][g]) = v;
          }
        char* cbase = reinterpret_cast<char*>(p.C + (int64_t)(j0 + wj * 128 + b * 32) * p.I + h0);
#pragma unroll
        for (int it = 0; it < 4; it++) {
          const int row = it * 8 + g_rq;
          const u32x4 v = *(const lds_u32x4*)(wtile + row * 256 + ((g_m ^ (row & 15)) << 4));
          if (RAG && j0 + wj * 128 + b * 32 + row >= p.J) continue;   // a row past the end
          if (p.cblocked) {
            // blocked output (the down projection reads it best that way): row R of the matrix, columns col .. col + 7
            const int64_t R = j0 + wj * 128 + b * 32 + row;
            const int col = h0 + g_m * 8;
            *reinterpret_cast<u32x4*>(p.C + (((R >> 5) * (p.I >> 5) + (col >> 5)) << 10) + ((R & 31) << 5) + (col & 31)) = v;
            continue;
          }
          *reinterpret_cast<u32x4*>(cbase + ((int64_t)row * p.I + g_m * 8) * 2) = v;
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else if (EPI == EPI_PARTIAL) {
      // fp32 partial sums of this reduction part, straight from the registers (wave-uniform base + lane offset)
      float* out = p.Cpart + (int64_t)part * p.J * p.I;
      const uint32_t pvoff = (uint32_t)(e_l32 * p.I + e_half * 4) * 4u;
#pragma unroll
      for (int b = 0; b < 4; b++) {
        char* obase = reinterpret_cast<char*>(out + (int64_t)(j0 + wj * 128 + b * 32) * p.I + i0 + wi * 128);
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int g = 0; g < 4; g++) {
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; e++) v[e] = acc[a][b][g * 4 + e];
            if (RAG && j0 + wj * 128 + b * 32 + e_l32 >= p.J) continue;                          // a row past the end
            if (CRAG && i0 + wi * 128 + a * 32 + g * 8 + e_half * 4 >= p.I) continue;            // 4 columns past the end
            *reinterpret_cast<f32x4*>(obase + (a * 32 + g * 8) * 4 + pvoff) = v;
          }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else if (EPI != EPI_F1) {
      // rounded to bf16 and stored (forward: the bias is in the accumulators since their start; the row statistics
      // are taken by the normalisation kernel)
#pragma unroll
      for (int b = 0; b < 4; b++) {
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int g = 0; g < 4; g++) {
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; e++)
              v[e] = (bf16_t)(EPI == EPI_RELU ? __builtin_fmaxf(acc[a][b][g * 4 + e], 0.0f) : acc[a][b][g * 4 + e]);
            *(lds_bf16x4*)(wtile + woff[a][g]) = v;
          }
        flush_rows(b);
        __builtin_amdgcn_sched_barrier(0);   // one block row at a time: keeps the accumulator copies in few registers
      }
    } else {
      // Z (bias included) rounded to bf16 and stored; A = GELU(stored Z); per output row j, mean and sum of squared
      // deviations of A over this wave's 128 columns: 64 values in the lane, 64 in lane ^ 32.
      const int stat_tile = (i0 + wi * 128) >> 7;
      // CRAG: columns of this wave's 128 that exist (a multiple of 4, wave-uniform); the others are masked out
      int nvalid = 128;
      if (CRAG) { nvalid = p.I - (i0 + wi * 128); nvalid = nvalid < 0 ? 0 : (nvalid > 128 ? 128 : nvalid); }
      const float inv_valid = 1.0f / (float)(nvalid > 0 ? nvalid : 1);
#pragma unroll
      for (int b = 0; b < 4; b++) {
        const int64_t j = jw + b * 32;
        float sum = 0.0f;
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int g = 0; g < 4; g++) {
            bf16x4 zs;
            const bool live = !CRAG || a * 32 + g * 8 + e_half * 4 < nvalid;
#pragma unroll
            for (int e = 0; e < 4; e++) {
              zs[e] = (bf16_t)acc[a][b][g * 4 + e];
              const float act = live ? gelu<float>((float)zs[e]) : 0.0f;
              acc[a][b][g * 4 + e] = act;
              sum += act;
            }
            *(lds_bf16x4*)(wtile + woff[a][g]) = zs;
          }
        sum += __shfl_xor(sum, 32, kWave);
        const float mean = sum * inv_valid;
        float m2 = 0.0f;
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const bool live = !CRAG || a * 32 + (r >> 2) * 8 + e_half * 4 < nvalid;
            const float d = live ? acc[a][b][r] - mean : 0.0f;
            m2 = __builtin_fmaf(d, d, m2);
          }
        m2 += __shfl_xor(m2, 32, kWave);
        if (e_half == 0 && (!RAG || j < p.J) && (!CRAG || nvalid > 0)) {
          f32x2 o; o[0] = mean; o[1] = m2;
          p.part[(int64_t)stat_tile * p.J + j] = o;
        }
        flush_rows(b);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    if (!has_next) break;
    L = Ln; tc = tn;
  }
  wait_dma<0>();   // the re-fetches issued during the last tile must land before the workgroup may retire
}

template <bool P_RM, bool Q_RM, int EPI, int BK, int NS, bool RAG, bool CRAG = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_bf16_kernel(FastParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  gemm_tile_loop<P_RM, Q_RM, EPI, BK, NS, RAG, CRAG>(p, smem, (int)blockIdx.x, (int)gridDim.x, (int)blockIdx.y);
}

// Two contractions in one launch: the dX product on the first na * (parts of its reduction) workgroups and the dW
// product on the rest (nb workgroups per part of its reduction); a split reduction writes fp32 partial sums.  For
// outputs so small that neither contraction has a tile for every compute unit - a dX with few column tiles, a small
// dW - the two together still fill the chip, where two launches in a row would each leave part of it idle.
template <int BK, int NS, int EPIA, int EPIB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_bf16_pair_kernel(FastParams pa, FastParams pb, int na, int nb) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int id = (int)blockIdx.x, a_all = na * pa.split;
  if (id < a_all) {
    gemm_tile_loop<true, false, EPIA, BK, NS, false>(pa, smem, id % na, na, id / na);
  } else {
    const int t = id - a_all;
    gemm_tile_loop<true, true, EPIB, BK, NS, false>(pb, smem, t % nb, nb, t / nb);
  }
}

// Sum split-reduction partials [split][n] fp32 -> bf16.
__global__ __launch_bounds__(256) void reduce_split_kernel(const float* __restrict__ part, int split, int64_t n,
                                                           bf16_t* __restrict__ out) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  f32x4 s = *reinterpret_cast<const f32x4*>(part + i);
  for (int k = 1; k < split; k++) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(part + (int64_t)k * n + i);
    s[0] += t[0]; s[1] += t[1]; s[2] += t[2]; s[3] += t[3];
  }
  bf16x4 o;
  o[0] = (bf16_t)s[0]; o[1] = (bf16_t)s[1]; o[2] = (bf16_t)s[2]; o[3] = (bf16_t)s[3];
  *reinterpret_cast<bf16x4*>(out + i) = o;
}

// dst [cols][rows] = src [rows][cols]^T in 64 x 64 tiles through LDS (rows, cols multiples of 64): both sides move
// 128-byte row segments.
// The tile of source rows r0 .. r0 + 63 lands in destination columns (r0 / 64) * tile_stride + col_off .. + 63 of a
// destination with pitch dst_ld (plain transposition: dst_ld = rows, tile_stride = 64, col_off = 0).
__global__ __launch_bounds__(256) void transpose64_kernel(const bf16_t* __restrict__ src, int64_t rows, int64_t cols,
                                                          bf16_t* __restrict__ dst, int64_t dst_ld, int tile_stride,
                                                          int col_off) {
  __shared__ unsigned short tile[64][66];
  const int64_t c0 = (int64_t)blockIdx.x * 64, r0 = (int64_t)blockIdx.y * 64;
  const int t = threadIdx.x, r = t >> 2, q = (t & 3) * 16;
  const unsigned short* sp = reinterpret_cast<const unsigned short*>(src) + (r0 + r) * cols + c0 + q;
  const u32x4 a = *reinterpret_cast<const u32x4*>(sp), b = *reinterpret_cast<const u32x4*>(sp + 8);
#pragma unroll
  for (int e = 0; e < 4; e++) {
    tile[r][q + 2 * e] = (unsigned short)(a[e] & 0xffffu); tile[r][q + 2 * e + 1] = (unsigned short)(a[e] >> 16);
    tile[r][q + 8 + 2 * e] = (unsigned short)(b[e] & 0xffffu); tile[r][q + 8 + 2 * e + 1] = (unsigned short)(b[e] >> 16);
  }
  __syncthreads();
  u32x4 o0, o1;
#pragma unroll
  for (int e = 0; e < 4; e++) {
    o0[e] = (uint32_t)tile[q + 2 * e][r] | ((uint32_t)tile[q + 2 * e + 1][r] << 16);
    o1[e] = (uint32_t)tile[q + 8 + 2 * e][r] | ((uint32_t)tile[q + 8 + 2 * e + 1][r] << 16);
  }
  unsigned short* dp = reinterpret_cast<unsigned short*>(dst) + (c0 + r) * dst_ld + (r0 / 64) * tile_stride + col_off + q;
  *reinterpret_cast<u32x4*>(dp) = o0;
  *reinterpret_cast<u32x4*>(dp + 8) = o1;
}

// Padded copy of the rows [row0, rows) of a row-major matrix: rows_out rows of the same pitch, zeros past the end.
// (256 rows for a ragged row count; one more where the kernel also reads past the end of every row - a reduction
// length rounded up - so that the last row's surplus stays inside the copy.)
__global__ __launch_bounds__(256) void copy_tail_rows_kernel(const bf16_t* __restrict__ src, int64_t rows, int64_t ld,
                                                             int64_t row0, bf16_t* __restrict__ dst, int rows_out) {
  const int64_t n8 = (int64_t)rows_out * ld / 8;   // ld is a multiple of 8 on this path
  for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < n8; v += (int64_t)gridDim.x * 256) {
    const int64_t r = (v * 8) / ld;
    u32x4 x = {0u, 0u, 0u, 0u};
    if (row0 + r < rows) x = *reinterpret_cast<const u32x4*>(src + row0 * ld + v * 8);
    *reinterpret_cast<u32x4*>(dst + v * 8) = x;
  }
}

// Zero-padded copy of a row-major matrix: dst [rows_out][cols_out] = src [rows][cols] (cols, cols_out multiples of 8).
__global__ __launch_bounds__(256) void pad_matrix_kernel(const bf16_t* __restrict__ src, int64_t rows, int64_t cols,
                                                         bf16_t* __restrict__ dst, int64_t rows_out, int64_t cols_out) {
  const int64_t vpr = cols_out / 8, n8 = rows_out * vpr;
  for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < n8; v += (int64_t)gridDim.x * 256) {
    const int64_t r = v / vpr, c = (v - r * vpr) * 8;
    u32x4 x = {0u, 0u, 0u, 0u};
    if (r < rows && c < cols) x = *reinterpret_cast<const u32x4*>(src + r * cols + c);
    *reinterpret_cast<u32x4*>(dst + r * cols_out + c) = x;
  }
}
__global__ __launch_bounds__(256) void pad_vector_kernel(const float* __restrict__ src, int64_t n, float* __restrict__ dst,
                                                         int64_t n_out) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_out; i += (int64_t)gridDim.x * 256)
    dst[i] = i < n ? src[i] : 0.0f;
}

template <bool P_RM, bool Q_RM, int EPI, int BK, int NS, bool RAG = false, bool CRAG = false>
void launch(FastParams p, hipStream_t s) {
  static OnceFlags configured;   // the dynamic LDS limit is raised once per kernel and device
  auto kern = gemm_bf16_kernel<P_RM, Q_RM, EPI, BK, NS, RAG, CRAG>;
  if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kLdsBytes, &configured)) return;
  DeviceInfo di;
  if (!device_info(&di)) return;
  // persistent: at most one workgroup per CU (the LDS footprint allows no more); a multiple of the die count
  // whenever the tile count is, so that every die gets the same number
  const int ntiles = p.tiles_i * p.tiles_j;
  int wgs = di.cus / p.split;
  if (wgs < di.xcds) wgs = di.xcds;
  if (wgs > ntiles) wgs = ntiles;
  p.xcds = 1;
  if (di.xcds > 1 && ntiles % di.xcds == 0 && wgs >= di.xcds) {
    wgs -= wgs % di.xcds;
    p.xcds = di.xcds;
  }
  const dim3 grid((unsigned)wgs, (unsigned)p.split);
  hipLaunchKernelGGL(kern, grid, dim3(256), kLdsBytes, s, p);
}

// Pipeline shape per contraction (slice width, stages): 64 x 2 or 32 x 4, both 128 KB of LDS.
#ifndef FDL_F1_BK
#define FDL_F1_BK 64
#endif
#ifndef FDL_B3_BK
#define FDL_B3_BK 32
#endif
#ifndef FDL_B4_BK
#define FDL_B4_BK 32
#endif
constexpr int kF1BK = FDL_F1_BK, kB3BK = FDL_B3_BK, kB4BK = FDL_B4_BK;
constexpr int stages_of(int bk) { return kLdsStages / (2 * kTile * bk * 2); }

// ragged_j: J may be any number from kMinRaggedRows up (F1, B3: J = M); otherwise a multiple of the tile
constexpr int64_t kMinRaggedRows = 128;
bool dims_ok(int64_t I, int64_t J, int64_t R, int bk, bool ragged_j = false) {
  const int64_t tj = (J + kTile - 1) / kTile;
  return I > 0 && J > 0 && R > 0 && I % kTile == 0 && (ragged_j ? J >= kMinRaggedRows : J % kTile == 0) &&
         R % (stages_of(bk) * bk) == 0 && I <= (1 << 24) && J <= (1 << 24) && (I / kTile) * tj <= (1 << 30);
}

}  // namespace

bool fast_f1_supported(int64_t M, int64_t K, int64_t N) { return dims_ok(N, M, K, kF1BK, true); }
bool fast_b3_supported(int64_t M, int64_t K, int64_t N) { return dims_ok(K, M, N, kB3BK, true); }
// dW on the fast kernel: the whole reduction if M is a whole number of pipeline rounds, else its first
// fast_b4_rows(M) rows (the caller adds the remaining rows' contribution)
int64_t fast_b4_rows(int64_t M) { const int64_t u = (int64_t)kB4BK * stages_of(kB4BK); return M / u * u; }
bool fast_b4_supported(int64_t M, int64_t K, int64_t N) {
  return fast_b4_rows(M) >= 128 && dims_ok(K, N, fast_b4_rows(M), kB4BK);
}
int fast_f1_stat_tile_w() { return 128; }
size_t fast_f1_tail_bytes(int64_t M, int64_t K) { return M % kTile ? (size_t)kTile * K * 2 : 0; }

// ---- padded mode: N and K multiples of 8 (16-byte rows) but not both multiples of the tile ----------------------
// The contractions then run on the same kernels with N and K rounded up to the tile: the weights are copied into a
// zero-padded [Np][Kp] matrix (small: it is the only operand that is copied whole), the bias into a padded vector,
// dZ is laid out with pitch Np and zero surplus columns, and the kernels leave the surplus output columns and rows
// unstored.  Where X is read past the end of its rows (K rounded up: forward) the surplus is the start of X's next
// row times the weights' zero padding; only X's last row has no next row, so the forward pass takes its last row tile
// from a copy with one spare row.
int64_t fast_pad_dim(int64_t n) { return (n + kTile - 1) / kTile * kTile; }
bool fast_padded_supported(int64_t M, int64_t K, int64_t N) {
  // K >= 128: a row read up to the rounded-up K then ends inside the next row (Kp <= 2 K), which is what keeps those
  // reads inside X (every row the kernels read that way has a successor) and inside the copy of X's last rows
  if (M < kMinRaggedRows || N < 8 || K < 128 || N % 8 || K % 8) return false;
  if (N % kTile == 0 && K % kTile == 0) return false;     // nothing to pad: the plain fast path applies
  const int64_t Np = fast_pad_dim(N), Kp = fast_pad_dim(K), tj = (M + kTile - 1) / kTile;
  return Np <= (1 << 24) && Kp <= (1 << 24) && M <= (1 << 24) && (Np / kTile) * tj <= (1 << 30) && (Kp / kTile) * tj <= (1 << 30) &&
         (Np / kTile) * (Kp / kTile) <= (1 << 30);
}
size_t fast_padded_tail_bytes(int64_t K) { return (size_t)(kTile + 1) * K * 2; }
// rows of the dW reduction the fast kernel covers in padded mode: where X is read past the end of its rows (K rounded
// up) the last row it touches must have a successor
int64_t fast_padded_b4_rows(int64_t M, int64_t K) {
  const int64_t u = (int64_t)kB4BK * stages_of(kB4BK);
  return (K % kTile ? M - 1 : M) / u * u;
}

// Wp [Np][Kp] and biasp [Np] (biasp and bias may be null) from W [N][K] and bias [N]
void launch_fast_pad_weights(int64_t K, int64_t N, const void* W, const float* bias, void* Wp, float* biasp, hipStream_t s) {
  const int64_t Np = fast_pad_dim(N), Kp = fast_pad_dim(K);
  const int64_t n8 = Np * Kp / 8;
  int64_t blocks = (n8 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(pad_matrix_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const bf16_t*)W, N, K, (bf16_t*)Wp, Np, Kp);
  if (biasp != nullptr)
    hipLaunchKernelGGL(pad_vector_kernel, dim3((unsigned)((Np + 255) / 256)), dim3(256), 0, s, bias, N, biasp, Np);
}

// Wt [K][N] = W^T (N, K multiples of 64).
void launch_fast_transpose(int64_t N, int64_t K, const void* W, void* Wt, hipStream_t s) {
  const dim3 grid((unsigned)(K / 64), (unsigned)(N / 64));
  hipLaunchKernelGGL(transpose64_kernel, grid, dim3(256), 0, s, (const bf16_t*)W, N, K, (bf16_t*)Wt, N, 64, 0);
}

// Wcat [D][2H]: the transposed gate and up weights side by side in groups of 64 columns - 64 of Wg^T, the same 64 of
// Wu^T, the next 64 of Wg^T, ... - which is the order in which the gated kernel wants the 256 rows of its P tile
// (H, D multiples of 64).
void launch_fast_transpose_gate(int64_t H, int64_t D, const void* Wg, const void* Wu, void* Wcat, hipStream_t s) {
  const dim3 grid((unsigned)(D / 64), (unsigned)(H / 64));
  hipLaunchKernelGGL(transpose64_kernel, grid, dim3(256), 0, s, (const bf16_t*)Wg, H, D, (bf16_t*)Wcat, 2 * H, 128, 0);
  hipLaunchKernelGGL(transpose64_kernel, grid, dim3(256), 0, s, (const bf16_t*)Wu, H, D, (bf16_t*)Wcat, 2 * H, 128, 64);
}

// part != nullptr: also emit the per-(row, 128-column tile) partial statistics of GELU(Zsave).
// xtail: fast_f1_tail_bytes(M, K) bytes of scratch for the padded copy of X's last rows (M not a multiple of 256)
// Wt: null, or W^T [K][N] (launch_fast_transpose): the weights then enter as the r-major operand.  A tile slice of an
// r-major operand is 32 runs of 512 contiguous bytes, of an r-contiguous one 256 runs of 128 or 64 bytes, and the
// contraction runs faster for every operand it can read the first way (measured on 65536 x 2048 x 8192: 1.77 -> 1.65
// ms; with the reduction long enough to hide the tile boundaries the three combinations reach 1.16 - 1.27, 1.31 - 1.35
// and 1.43 - 1.44 PFLOP/s), which pays for transposing the weights once the batch is large (the caller decides).
void launch_fast_f1(int64_t M, int64_t K, int64_t N, const void* X, const void* W, const void* Wt, const float* bias,
                    void* Zsave, void* part, void* xtail, hipStream_t s) {
  FastParams p = {};
  p.P = (const bf16_t*)W; p.Q = (const bf16_t*)X; p.ldp = K; p.ldq = K;
  p.C = (bf16_t*)Zsave; p.bias = bias; p.part = (f32x2*)part;
  p.I = (int)N; p.J = (int)M; p.tiles_i = (int)(N / kTile); p.tiles_j = (int)((M + kTile - 1) / kTile);
  p.nkt = (int)(K / kF1BK); p.split = 1;
  const bool rag = M % kTile != 0;
  if (rag) {
    p.Qtail = (const bf16_t*)xtail;
    hipLaunchKernelGGL(copy_tail_rows_kernel, dim3(64), dim3(256), 0, s, (const bf16_t*)X, M, K,
                       (int64_t)(p.tiles_j - 1) * kTile, (bf16_t*)xtail, kTile);
  }
  if (Wt != nullptr) {
    p.P = (const bf16_t*)Wt; p.ldp = N; p.nkt = (int)(K / kB3BK);
    constexpr int NS = stages_of(kB3BK);
    if (rag) {
      if (part != nullptr) launch<true, false, EPI_F1, kB3BK, NS, true>(p, s);
      else launch<true, false, EPI_BIAS, kB3BK, NS, true>(p, s);
    } else {
      if (part != nullptr) launch<true, false, EPI_F1, kB3BK, NS>(p, s);
      else launch<true, false, EPI_BIAS, kB3BK, NS>(p, s);
    }
    return;
  }
  if (rag) {
    if (part != nullptr) launch<false, false, EPI_F1, kF1BK, stages_of(kF1BK), true>(p, s);
    else launch<false, false, EPI_BIAS, kF1BK, stages_of(kF1BK), true>(p, s);
  } else {
    if (part != nullptr) launch<false, false, EPI_F1, kF1BK, stages_of(kF1BK)>(p, s);
    else launch<false, false, EPI_BIAS, kF1BK, stages_of(kF1BK)>(p, s);
  }
}

// Padded mode: Wp [Np][Kp], biasp [Np] from launch_fast_pad_weights; xtail: fast_padded_tail_bytes(K) bytes
void launch_fast_f1_padded(int64_t M, int64_t K, int64_t N, const void* X, const void* Wp, const float* biasp, void* Zsave,
                           void* part, void* xtail, hipStream_t s) {
  const int64_t Np = fast_pad_dim(N), Kp = fast_pad_dim(K);
  FastParams p = {};
  p.P = (const bf16_t*)Wp; p.Q = (const bf16_t*)X; p.ldp = Kp; p.ldq = K;
  p.C = (bf16_t*)Zsave; p.bias = biasp; p.part = (f32x2*)part;
  p.I = (int)N; p.J = (int)M; p.tiles_i = (int)(Np / kTile); p.tiles_j = (int)((M + kTile - 1) / kTile);
  p.nkt = (int)(Kp / kF1BK); p.split = 1;
  // the last row tile always comes from the copy: its rows are read up to Kp columns, and X's last row has no successor
  p.Qtail = (const bf16_t*)xtail;
  hipLaunchKernelGGL(copy_tail_rows_kernel, dim3(64), dim3(256), 0, s, (const bf16_t*)X, M, K,
                     (int64_t)(p.tiles_j - 1) * kTile, (bf16_t*)xtail, kTile + 1);
  if (part != nullptr) launch<false, false, EPI_F1, kF1BK, stages_of(kF1BK), true, true>(p, s);
  else launch<false, false, EPI_BIAS, kF1BK, stages_of(kF1BK), true, true>(p, s);
}

// out[m][n] = f(sum_k X[m][k] W[n][k] + bias[n]) for the sibling operators; same shape rules as launch_fast_f1.
//   kind 0: plain product (bias may be null: then none is added)      kind 1: max(. , 0)
//   kind 2: aux[m][n] where the sum is positive, else 0
// xtail: fast_f1_tail_bytes(M, K) bytes of scratch when M is not a multiple of 256, unless X itself has readable rows
// up to the next multiple of 256 (x_padded).  Wt: null, or W^T [K][N] from launch_fast_transpose.
// out_blocked (kind 2 only; M, N multiples of 32): out is written in 32 x 32 blocks, as the dX and dW kernels read it best.
void launch_fast_xwt(int kind, int64_t M, int64_t K, int64_t N, const void* X, bool x_padded, const void* W,
                     const void* Wt, const float* bias, const void* aux, void* out, bool out_blocked, void* xtail,
                     hipStream_t s, bool x_blocked) {
  FastParams p = {};
  p.cblocked = (out_blocked && kind == 2) ? 1 : 0;
  p.qblocked = (x_blocked && Wt != nullptr) ? 1 : 0;   // only the transposed-weight kernels read a blocked X
  p.P = (const bf16_t*)W; p.Q = (const bf16_t*)X; p.ldp = K; p.ldq = K;
  p.C = (bf16_t*)out; p.bias = bias; p.aux = (const bf16_t*)aux;
  p.I = (int)N; p.J = (int)M; p.tiles_i = (int)(N / kTile); p.tiles_j = (int)((M + kTile - 1) / kTile);
  p.nkt = (int)(K / kF1BK); p.split = 1;
  const bool rag = M % kTile != 0;
  if (rag && !x_padded) {
    p.Qtail = (const bf16_t*)xtail;
    hipLaunchKernelGGL(copy_tail_rows_kernel, dim3(64), dim3(256), 0, s, (const bf16_t*)X, M, K,
                       (int64_t)(p.tiles_j - 1) * kTile, (bf16_t*)xtail, kTile);
  }
  if (Wt != nullptr) {   // the weights as the r-major operand (see launch_fast_f1)
    p.P = (const bf16_t*)Wt; p.ldp = N; p.nkt = (int)(K / kB3BK);
    constexpr int NST = stages_of(kB3BK);
#define FDL_XWT_T(EPI)                                                            \
  do {                                                                            \
    if (rag) launch<true, false, EPI, kB3BK, NST, true>(p, s);                    \
    else launch<true, false, EPI, kB3BK, NST, false>(p, s);                       \
  } while (0)
    if (kind == 1) FDL_XWT_T(EPI_RELU);
    else if (kind == 2) FDL_XWT_T(EPI_MASK);
    else if (bias != nullptr) FDL_XWT_T(EPI_BIAS);
    else FDL_XWT_T(EPI_STORE);
#undef FDL_XWT_T
    return;
  }
  constexpr int NS = stages_of(kF1BK);
#define FDL_XWT(EPI)                                                              \
  do {                                                                            \
    if (rag) launch<false, false, EPI, kF1BK, NS, true>(p, s);                    \
    else launch<false, false, EPI, kF1BK, NS, false>(p, s);                       \
  } while (0)
  if (kind == 1) FDL_XWT(EPI_RELU);
  else if (kind == 2) FDL_XWT(EPI_MASK);
  else if (bias != nullptr) FDL_XWT(EPI_BIAS);
  else FDL_XWT(EPI_STORE);
#undef FDL_XWT
}

// Gated pair of products for the feed-forward block: Hout[m][h] = SiLU(sum_d X[m][d] Wg[h][d]) * (sum_d X[m][d] Wu[h][d]).
// Shapes: H a multiple of 128, D of the pipeline round, M >= 128; ragged M as in launch_fast_xwt.
bool fast_gate_supported(int64_t M, int64_t D, int64_t H) {
  const int64_t tj = (M + kTile - 1) / kTile;
  return M >= kMinRaggedRows && H > 0 && H % 128 == 0 && D > 0 && D % (stages_of(kF1BK) * kF1BK) == 0 && H <= (1 << 24) &&
         M <= (1 << 24) && (H / 128) * tj <= (1 << 30);
}
void launch_fast_gate(int64_t M, int64_t D, int64_t H, const void* X, const void* Wg, const void* Wu, const void* Wcat,
                      void* Hout, bool out_blocked, void* xtail, hipStream_t s) {
  FastParams p = {};
  p.cblocked = out_blocked ? 1 : 0;    // H a multiple of 32; rows past M are not stored
  p.P = (const bf16_t*)Wg; p.P2 = (const bf16_t*)Wu; p.Q = (const bf16_t*)X; p.ldp = D; p.ldq = D;
  p.C = (bf16_t*)Hout;
  p.I = (int)H; p.J = (int)M; p.tiles_i = (int)(H / 128); p.tiles_j = (int)((M + kTile - 1) / kTile);
  p.nkt = (int)(D / kF1BK); p.split = 1;
  const bool rag = M % kTile != 0;
  if (rag) {
    p.Qtail = (const bf16_t*)xtail;
    hipLaunchKernelGGL(copy_tail_rows_kernel, dim3(64), dim3(256), 0, s, (const bf16_t*)X, M, D,
                       (int64_t)(p.tiles_j - 1) * kTile, (bf16_t*)xtail, kTile);
  }
  if (Wcat != nullptr) {   // Wcat from launch_fast_transpose_gate: the weights as one r-major operand (see launch_fast_f1)
    p.P = (const bf16_t*)Wcat; p.P2 = nullptr; p.ldp = 2 * H; p.nkt = (int)(D / kB3BK);
    constexpr int NST = stages_of(kB3BK);
    if (rag) launch<true, false, EPI_GATE, kB3BK, NST, true>(p, s);
    else launch<true, false, EPI_GATE, kB3BK, NST, false>(p, s);
    return;
  }
  constexpr int NS = stages_of(kF1BK);
  if (rag) launch<false, false, EPI_GATE, kF1BK, NS, true>(p, s);
  else launch<false, false, EPI_GATE, kF1BK, NS, false>(p, s);
}

void launch_fast_b3(int64_t M, int64_t K, int64_t N, const void* dZ, bool dz_blocked, const void* W, void* dX,
                    hipStream_t s) {
  FastParams p = {};
  p.qblocked = dz_blocked ? 1 : 0;
  p.P = (const bf16_t*)W; p.Q = (const bf16_t*)dZ; p.ldp = K; p.ldq = N;
  p.C = (bf16_t*)dX;
  p.I = (int)K; p.J = (int)M; p.tiles_i = (int)(K / kTile); p.tiles_j = (int)((M + kTile - 1) / kTile);
  p.nkt = (int)(N / kB3BK); p.split = 1;
  // ragged M: dZ is the library's own buffer and has readable rows up to the end of the last row tile
  if (M % kTile) launch<true, false, EPI_STORE, kB3BK, stages_of(kB3BK), true>(p, s);
  else launch<true, false, EPI_STORE, kB3BK, stages_of(kB3BK)>(p, s);
}

// Padded mode: dZ [.][Np] with zero surplus columns and readable rows up to the next multiple of 256; Wp [Np][Kp]
void launch_fast_b3_padded(int64_t M, int64_t K, int64_t N, const void* dZ, const void* Wp, void* dX, hipStream_t s) {
  const int64_t Np = fast_pad_dim(N), Kp = fast_pad_dim(K);
  FastParams p = {};
  p.P = (const bf16_t*)Wp; p.Q = (const bf16_t*)dZ; p.ldp = Kp; p.ldq = Np;
  p.C = (bf16_t*)dX;
  p.I = (int)K; p.J = (int)M; p.tiles_i = (int)(Kp / kTile); p.tiles_j = (int)((M + kTile - 1) / kTile);
  p.nkt = (int)(Np / kB3BK); p.split = 1;
  launch<true, false, EPI_STORE, kB3BK, stages_of(kB3BK), true, true>(p, s);
}

// Split of the reduction over M.  One workgroup per compute unit walks the (tile, part) units of its part, so the
// kernel takes ceil(tiles * split / CUs) rounds of M / split rows each: a small dW fills the chip only when split,
// and a dW with a few tiles more than a whole number of rounds (9 x 32 = 288 tiles on 256 compute units: two rounds,
// the second nearly empty) loses up to half its time unless the rounds are made shorter.  Against that stands the
// traffic of the fp32 partial sums (written, read again and summed).  Both are priced with round figures for this
// part - 23 ns per reduction row and round, 4 TB/s for the partial sums - and the cheapest split wins; each part keeps
// at least 512 rows and a whole number of pipeline rounds, and the partial sums at most 512 MB.
int fast_b4_split(int64_t M, int64_t K, int64_t N) {
  const int64_t tiles = ((K + kTile - 1) / kTile) * ((N + kTile - 1) / kTile);
  const int64_t unit = (int64_t)kB4BK * stages_of(kB4BK);   // every part is a whole number of slice groups
  int best = 1;
  double best_cost = 0.0;
  for (int split = 1; split <= 16; split *= 2) {
    if (split > 1 && (M % (split * unit) != 0 || M / split < 512)) break;
    const double partial_bytes = split > 1 ? (double)split * (double)tiles * kTile * kTile * 4.0 : 0.0;
    if (partial_bytes > 512.0 * 1024 * 1024) break;
    const int64_t rounds = (tiles * split + kPlanCUs - 1) / kPlanCUs;
    const double cost = (double)rounds * (double)(M / split) * 23e-9 + 2.0 * partial_bytes / 4e12;
    if (split == 1 || cost < 0.97 * best_cost) { best = split; best_cost = cost; }
  }
  return best;   // M: the rows the fast kernel covers
}

// dW from the first M rows (a whole number of pipeline rounds, see fast_b4_rows).  With split > 1 or extra > 0 the
// kernel writes fp32 partial sums dwpart[0 .. split); the caller may add `extra` more partials behind them (the
// rows the fast kernel does not cover) and then sums them (launch_fast_b4_reduce, or the backward pass's finishing
// launch); otherwise dW is final on return.
void launch_fast_b4(int64_t M, int64_t K, int64_t N, int split, int extra, const void* dZ, bool dz_blocked, const void* X,
                    void* dW, void* dwpart, hipStream_t s) {
  FastParams p = {};
  p.qblocked = dz_blocked ? 1 : 0;
  p.P = (const bf16_t*)X; p.Q = (const bf16_t*)dZ; p.ldp = K; p.ldq = N;
  p.C = (bf16_t*)dW; p.Cpart = (float*)dwpart;
  p.I = (int)K; p.J = (int)N; p.tiles_i = (int)(K / kTile); p.tiles_j = (int)(N / kTile);
  p.nkt = (int)(M / kB4BK / split); p.split = split;
  if (split > 1 || extra > 0) launch<true, true, EPI_PARTIAL, kB4BK, stages_of(kB4BK)>(p, s);
  else launch<true, true, EPI_STORE, kB4BK, stages_of(kB4BK)>(p, s);
}

// Padded mode: dZ has pitch Np (zero surplus columns); X is read up to Kp columns per row, so M must be at most
// fast_padded_b4_rows.  Always writes fp32 partial sums dwpart[0 .. split) (pitch K, surplus rows and columns unstored);
// the caller adds what it must and calls launch_fast_b4_reduce.
void launch_fast_b4_padded(int64_t M, int64_t K, int64_t N, int split, const void* dZ, const void* X, void* dwpart,
                           hipStream_t s) {
  const int64_t Np = fast_pad_dim(N), Kp = fast_pad_dim(K);
  FastParams p = {};
  p.P = (const bf16_t*)X; p.Q = (const bf16_t*)dZ; p.ldp = K; p.ldq = Np;
  p.C = nullptr; p.Cpart = (float*)dwpart;
  p.I = (int)K; p.J = (int)N; p.tiles_i = (int)(Kp / kTile); p.tiles_j = (int)(Np / kTile);
  p.nkt = (int)(M / kB4BK / split); p.split = split;
  launch<true, true, EPI_PARTIAL, kB4BK, stages_of(kB4BK), true, true>(p, s);
}

void launch_fast_b4_reduce(int64_t K, int64_t N, int parts, const void* dwpart, void* dW, hipStream_t s) {
  const int64_t n = N * K;
  hipLaunchKernelGGL(reduce_split_kernel, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, s,
                     (const float*)dwpart, parts, n, (bf16_t*)dW);
}

// dX and dW in one launch (see gemm_bf16_pair_kernel): for shapes where every dimension is a whole number of tiles and
// the two outputs together have at most one tile per compute unit of the plan's part (kPlanCUs: the split is part of
// the workspace plan and must not depend on the device).  The reductions (over N for dX, over M for dW) are split into
// sa and sb parts - whole pipeline rounds of at least 512 - so that the workgroups fill the chip and the longer of the
// two kinds of workgroup is as short as possible.  Returns false if the shape does not qualify.
bool fast_pair_plan(int64_t M, int64_t K, int64_t N, int* sa_out, int* sb_out) {
  if (static_cast<int>(kB3BK) != static_cast<int>(kB4BK)) return false;
  if (M % kTile || !dims_ok(K, M, N, kB3BK) || !dims_ok(K, N, M, kB4BK)) return false;
  const int64_t ta = (K / kTile) * (M / kTile), tb = (K / kTile) * (N / kTile);
  if (ta + tb > kPlanCUs) return false;
  const int64_t unit = (int64_t)kB3BK * stages_of(kB3BK);
  int best_sa = 0, best_sb = 0;
  int64_t best_len = 0, best_wgs = 0;
  for (int sa = 1; sa <= 16; sa *= 2) {
    if (N % (sa * unit) || (sa > 1 && N / sa < 512)) break;
    for (int sb = 1; sb <= 16; sb *= 2) {
      if (M % (sb * unit) || (sb > 1 && M / sb < 512)) break;
      const int64_t wgs = ta * sa + tb * sb;
      if (wgs > kPlanCUs) break;
      const int64_t len = N / sa > M / sb ? N / sa : M / sb;     // reduction length of the longest workgroup
      if (best_sa == 0 || len < best_len || (len == best_len && wgs < best_wgs)) {
        best_sa = sa; best_sb = sb; best_len = len; best_wgs = wgs;
      }
    }
  }
  if (best_sa == 0) return false;
  *sa_out = best_sa; *sb_out = best_sb;
  return true;
}

// dxpart: sa [M][K] fp32 partial sums (sa > 1), dwpart: sb [N][K] (sb > 1); an unsplit product goes to dX / dW directly.
// The caller sums the partials (launch_fast_b4_reduce works for either).
void launch_fast_pair(int64_t M, int64_t K, int64_t N, int sa, int sb, const void* dZ, bool dz_blocked, const void* W,
                      const void* X, void* dX, void* dxpart, void* dW, void* dwpart, hipStream_t s) {
  FastParams pa = {}, pb = {};
  pa.qblocked = pb.qblocked = dz_blocked ? 1 : 0;
  pa.P = (const bf16_t*)W; pa.Q = (const bf16_t*)dZ; pa.ldp = K; pa.ldq = N; pa.C = (bf16_t*)dX; pa.Cpart = (float*)dxpart;
  pa.I = (int)K; pa.J = (int)M; pa.tiles_i = (int)(K / kTile); pa.tiles_j = (int)(M / kTile);
  pa.nkt = (int)(N / kB3BK / sa); pa.split = sa;
  pb.P = (const bf16_t*)X; pb.Q = (const bf16_t*)dZ; pb.ldp = K; pb.ldq = N; pb.C = (bf16_t*)dW; pb.Cpart = (float*)dwpart;
  pb.I = (int)K; pb.J = (int)N; pb.tiles_i = (int)(K / kTile); pb.tiles_j = (int)(N / kTile);
  pb.nkt = (int)(M / kB4BK / sb); pb.split = sb;
  DeviceInfo di;
  if (!device_info(&di)) return;
  const int na = pa.tiles_i * pa.tiles_j, nb = pb.tiles_i * pb.tiles_j;     // one tile per workgroup
  const bool die_aware = di.xcds > 1 && na % di.xcds == 0 && nb % di.xcds == 0;
  pa.xcds = die_aware ? di.xcds : 1; pb.xcds = pa.xcds;
  const dim3 grid((unsigned)(na * sa + nb * sb));
  constexpr int NS = stages_of(kB3BK);
#define FDL_PAIR(EA, EB)                                                                                   \
  do {                                                                                                     \
    static OnceFlags configured;                                                                           \
    auto kern = gemm_bf16_pair_kernel<kB3BK, NS, EA, EB>;                                                  \
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), kLdsBytes, &configured)) return;          \
    hipLaunchKernelGGL(kern, grid, dim3(256), kLdsBytes, s, pa, pb, na, nb);                               \
  } while (0)
  if (sa > 1 && sb > 1) FDL_PAIR(EPI_PARTIAL, EPI_PARTIAL);
  else if (sa > 1) FDL_PAIR(EPI_PARTIAL, EPI_STORE);
  else if (sb > 1) FDL_PAIR(EPI_STORE, EPI_PARTIAL);
  else FDL_PAIR(EPI_STORE, EPI_STORE);
#undef FDL_PAIR
}

}  // namespace fdl
