// bf16 MFMA GEMM for the three contractions of the fused dense-layer block (gfx950).
//
//     D[i][j] = sum_r P(i,r) * Q(j,r)      stored as C[j][i]   (C row-major, leading dimension I)
//
// P feeds the MFMA "A" side, Q the "B" side, so a lane ends up with 4 consecutive i (output columns) of one
// output row j in adjacent accumulator registers: rows of C are written with 8-byte stores, and a row
// reduction over i (the LayerNorm statistics of the forward pass) is a sum inside the lane plus one
// cross-half exchange.
//
//   F1  Z[m][n]  = sum_k X[m][k] W[n][k] + b[n]   P = W (i = n, r-contiguous)   Q = X  (j = m, r-contiguous)
//   B3  dX[m][k] = sum_n dZ[m][n] W[n][k]         P = W (i = k, r = n major)    Q = dZ (j = m, r-contiguous)
//   B4  dW[n][k] = sum_m dZ[m][n] X[m][k]         P = X (i = k, r = m major)    Q = dZ (j = n, r = m major)
// (the linear layer's forward, grad-input and grad-weight products of the paper's linear tasks.)
//
// Workgroup: 256 threads = 4 waves (2 x 2), one per SIMD; block tile 256 x 256, wave tile 128 x 128 as 4 x 4
// v_mfma_f32_32x32x16_bf16 blocks (256 fp32 accumulators per lane, held in AGPRs); reduction slices of 64, two
// LDS stages of 64 KB filled by direct global->LDS loads (16 bytes per lane, no staging registers) that stay in
// flight for a whole slice time while the MFMAs of the other stage run.
//
// LDS tile layouts (both XOR-swizzled by choosing which global chunk a lane fetches, since a direct load
// lands at base + lane*16):
//   r-contiguous operand: [256 rows][8 chunks of 16 B]; chunk c of row w sits in slot c ^ (w & 7); fragments
//       are read with ds_read_b128 (8 consecutive r for the lane's row).
//   r-major operand:      [64 r-rows][32 chunks of 16 B]; chunk c of r-row w sits in slot c ^ ((w & 3) << 1);
//       fragments are read with the transposing ds_read_b64_tr_b16 (4 consecutive r for the lane's column).
#include "common.hip.h"
#include "internal.h"

namespace fdl {
namespace {

constexpr int kTile = 256;
constexpr int kBK = 64;
constexpr int kOperandBytes = kTile * kBK * 2;   // 32 KB
constexpr int kStageBytes = 2 * kOperandBytes;   // 64 KB
constexpr int kLdsBytes = 2 * kStageBytes;       // 128 KB

enum { EPI_STORE = 0, EPI_F1 = 1 };

struct FastParams {
  const bf16_t* P; const bf16_t* Q;
  int64_t ldp, ldq;
  bf16_t* C;             // [J][I]
  float* Cpart;          // [split][J][I] fp32 (split > 1)
  const float* bias;     // [I]   (EPI_F1)
  f32x2* part;           // [I/128][J]  (EPI_F1)
  int I, J;
  int tiles_i, tiles_j;
  int nkt;               // reduction slices per workgroup
  int split;
};

typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((ext_vector_type(4))) short short4_;
typedef __attribute__((address_space(3))) short4_ lds_short4;

// 16 bytes per lane, global -> LDS, no registers: lane l's data lands at (lds_base + LDS_OFF) + 16 l.
// voff: per-lane byte offset, sbase: wave-uniform global base, lds_base: wave-uniform LDS byte address.
// M0 carries the LDS address; one wait state separates the SALU write of M0 from the load that reads it.
template <int LDS_OFF>
__device__ __forceinline__ void dma16(uint32_t voff, const void* sbase, uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(sbase), "s"(lds_base), "n"(LDS_OFF) : "memory", "m0", "scc");
}
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <bool RM> struct Loader {
  // voff[q]: per-lane byte offset of instruction q (constant over the reduction loop).  Eight instructions per
  // wave fill this wave's quarter of the 32 KB operand tile; the only per-slice scalar work is one base pointer.
  uint32_t voff[8];
  __device__ __forceinline__ void init(int lane, int64_t ld) {
#pragma unroll
    for (int q = 0; q < 8; q++) {
      if (RM) {
        // instruction q covers r-rows 2q, 2q+1 (of this wave's 16); lane: r-row 2q + h, h = lane/32, slot lane%32
        const int h = lane >> 5, slot = lane & 31;
        const int c = slot ^ (((2 * q + h) & 3) << 1);
        voff[q] = (uint32_t)((int64_t)(2 * q + h) * ld * 2 + c * 16);
      } else {
        // instruction q covers rows 8q..8q+7 (of this wave's 64); lane: row 8q + w, w = lane/8, slot lane%8
        const int w = lane >> 3, slot = lane & 7;
        voff[q] = (uint32_t)((int64_t)(8 * q + w) * ld * 2 + ((slot ^ w) * 16));
      }
    }
  }
  // first element this wave fetches of the slice that starts at `base` (block tile origin, first r of the slice)
  __device__ __forceinline__ const bf16_t* wave_base(const bf16_t* base, int64_t ld, int wave) const {
    return RM ? base + (int64_t)(wave * 16) * ld : base + (int64_t)(wave * 64) * ld;
  }
  // wbase: wave_base(...) of the slice; wlds: LDS address of this wave's quarter of the operand tile
  template <int Q> __device__ __forceinline__ void issue1(const bf16_t* wbase, uint32_t wlds) const {
    dma16<Q * 1024>(voff[Q], wbase, wlds);
  }
  // q is a compile-time constant at every call site once the surrounding loop is unrolled
  __device__ __forceinline__ void issue_q(int q, const bf16_t* wbase, uint32_t wlds) const {
    switch (q) {
      case 0: issue1<0>(wbase, wlds); break;
      case 1: issue1<1>(wbase, wlds); break;
      case 2: issue1<2>(wbase, wlds); break;
      case 3: issue1<3>(wbase, wlds); break;
      case 4: issue1<4>(wbase, wlds); break;
      case 5: issue1<5>(wbase, wlds); break;
      case 6: issue1<6>(wbase, wlds); break;
      default: issue1<7>(wbase, wlds); break;
    }
  }
  __device__ __forceinline__ void issue(const bf16_t* wbase, uint32_t wlds) const {
    issue1<0>(wbase, wlds); issue1<1>(wbase, wlds); issue1<2>(wbase, wlds); issue1<3>(wbase, wlds);
    issue1<4>(wbase, wlds); issue1<5>(wbase, wlds); issue1<6>(wbase, wlds); issue1<7>(wbase, wlds);
  }
};

template <bool RM> struct Frags {
  // LDS byte offsets of this lane's fragment reads inside an operand tile.
  //  r-contiguous: off[kk] for the 4 sub-slices; block a adds a*4096 (32 rows of 128 B).
  //  r-major:      off[a] for the 4 blocks; sub-slice kk and half t add (kk*16 + 4t)*512.
  uint32_t off[4];
  __device__ __forceinline__ void init(int lane, int w /* wave coordinate along this operand */) {
    if (RM) {
      const int G = lane >> 4, p = lane & 15;
      const int r = 8 * (G >> 1) + (p >> 2);
#pragma unroll
      for (int a = 0; a < 4; a++) {
        const int c = w * 16 + a * 4 + 2 * (G & 1) + ((p & 3) >> 1);
        off[a] = (uint32_t)(r * 512 + ((c ^ ((p >> 2) << 1)) * 16) + (p & 1) * 8);
      }
    } else {
      const int row = w * 128 + (lane & 31);
      const int t0 = (lane >> 5) ^ (lane & 7);
#pragma unroll
      for (int kk = 0; kk < 4; kk++) off[kk] = (uint32_t)(row * 128 + (((kk << 1) ^ t0) << 4));
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
      return *(const lds_bf16x8*)(tile + off[kk] + a * 4096);
    }
  }
};

template <bool P_RM, bool Q_RM, int EPI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_bf16_kernel(FastParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const lds_char* lds = (const lds_char*)smem;
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wi = wave & 1, wj = wave >> 1;

  // ---- workgroup -> tile: consecutive ids on one XCD (ids are dealt round-robin over the 8 XCDs) walk a band
  // of 8 output-row tiles, so the 32 workgroups resident on an XCD share 4 P panels and 8 Q panels in its L2.
  const int ntiles = p.tiles_i * p.tiles_j;
  int L = blockIdx.x;
  if ((ntiles & 7) == 0) L = (blockIdx.x & 7) * (ntiles >> 3) + (blockIdx.x >> 3);
  const int band_tiles = 8 * p.tiles_i;
  const int band = L / band_tiles;
  const int rem = L - band * band_tiles;
  int band_h = p.tiles_j - band * 8;
  if (band_h > 8) band_h = 8;
  const int ti = rem / band_h;
  const int tj = band * 8 + rem % band_h;
  const int i0 = ti * kTile, j0 = tj * kTile;
  const int64_t r_begin = (int64_t)blockIdx.y * p.nkt * kBK;

  Loader<P_RM> lp; lp.init(lane, p.ldp);
  Loader<Q_RM> lq; lq.init(lane, p.ldq);
  Frags<P_RM> fp; fp.init(lane, wi);
  Frags<Q_RM> fq; fq.init(lane, wj);

  const bf16_t* pbase = P_RM ? p.P + r_begin * p.ldp + i0 : p.P + (int64_t)i0 * p.ldp + r_begin;
  const bf16_t* qbase = Q_RM ? p.Q + r_begin * p.ldq + j0 : p.Q + (int64_t)j0 * p.ldq + r_begin;
  const int64_t pstep = P_RM ? (int64_t)kBK * p.ldp : kBK;
  const int64_t qstep = Q_RM ? (int64_t)kBK * p.ldq : kBK;

  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; a++)
#pragma unroll
    for (int b = 0; b < 4; b++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[a][b][r] = 0.0f;

  const int last = p.nkt - 1;
  const uint32_t wlds = lds0 + (uint32_t)wave * 8192u;      // this wave's quarter of an operand tile
  lp.issue(lp.wave_base(pbase, p.ldp, wave), wlds);
  lq.issue(lq.wave_base(qbase, p.ldq, wave), wlds + kOperandBytes);
  {
    const int k1 = 1 < last ? 1 : last;
    lp.issue(lp.wave_base(pbase + k1 * pstep, p.ldp, wave), wlds + kStageBytes);
    lq.issue(lq.wave_base(qbase + k1 * qstep, p.ldq, wave), wlds + kStageBytes + kOperandBytes);
  }
  wait_dma();
  __syncthreads();

  // Fragments are double-buffered in registers: while the 16 MFMAs of sub-slice kk run, the 8 fragment reads of
  // sub-slice kk+1 are issued between them.  The last sub-slice's MFMAs are issued after the barrier that
  // publishes the next stage, behind the first fragment reads of that stage, so the matrix pipe has work while
  // those reads are in flight.
  bf16x8 pf[2][4], qf[2][4];
#pragma unroll
  for (int a = 0; a < 4; a++) pf[0][a] = fp.load(lds, a, 0);
#pragma unroll
  for (int b = 0; b < 4; b++) qf[0][b] = fq.load(lds + kOperandBytes, b, 0);

  for (int kt = 0; kt < p.nkt; kt++) {
    const int cur = kt & 1;
    // Slice kt+2 is fetched into this slice's own stage as soon as the barrier below has shown that every wave
    // holds its last fragments of slice kt in registers: the direct loads then have one whole slice time (the
    // most two stages allow) before the next barrier needs them.  Slices past the end are clamped to the last
    // one (fetched again, never read) so that the loop body is branch-free.
    const int k2 = kt + 2 < last ? kt + 2 : last;
    const uint32_t own = wlds + (uint32_t)cur * kStageBytes;
    const bf16_t* pn = lp.wave_base(pbase + (int64_t)k2 * pstep, p.ldp, wave);
    const bf16_t* qn = lq.wave_base(qbase + (int64_t)k2 * qstep, p.ldq, wave);
    const lds_char* tp = lds + cur * kStageBytes;
    const lds_char* tq = tp + kOperandBytes;
    const lds_char* np_ = lds + (cur ^ 1) * kStageBytes;
    const lds_char* nq_ = np_ + kOperandBytes;
    // Issue order is pinned by hand (a scheduling barrier after every step): MFMA t of a sub-slice is followed by
    // a fragment read of the next sub-slice (even t) and, in the last sub-slice, by one direct load, so neither
    // the LDS reads nor the global loads keep the matrix pipe waiting for long.
#pragma unroll
    for (int kk = 0; kk < 4; kk++) {
      const int use = kk & 1, fill = use ^ 1;
      if (kk == 3) {
        wait_dma();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
      const lds_char* rp = kk < 3 ? tp : np_;
      const lds_char* rq = kk < 3 ? tq : nq_;
      const int rk = kk < 3 ? kk + 1 : 0;
#pragma unroll
      for (int t = 0; t < 16; t++) {
        const int a = t >> 2, b = t & 3;
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[use][a], qf[use][b], acc[a][b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if ((t & 1) == 0) {
          // read order: P0, Q0, Q1, Q2, Q3, P1, P2, P3 (the order in which the next sub-slice consumes them)
          const int slot = t >> 1;
          if (slot == 0) pf[fill][0] = fp.load(rp, 0, rk);
          else if (slot <= 4) qf[fill][slot - 1] = fq.load(rq, slot - 1, rk);
          else pf[fill][slot - 4] = fp.load(rp, slot - 4, rk);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (kk == 3) {
          if (t < 8) lp.issue_q(t, pn, own);
          else lq.issue_q(t - 8, qn, own + kOperandBytes);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
  wait_dma();   // the clamped re-fetches of the last two iterations must land before the workgroup may retire

  // ------------------------------------------------------------------ epilogue
  // accumulator register r of block (a, b): i = a*32 + (r/4)*8 + (lane/32)*4 + r%4, j = b*32 + lane%32
  const int half = lane >> 5, l32 = lane & 31;
  const int iw = i0 + wi * 128 + half * 4;     // + a*32 + g*8 + e
  const int jw = j0 + wj * 128 + l32;          // + b*32
  if (EPI == EPI_STORE) {
    if (p.split > 1) {
      float* out = p.Cpart + (int64_t)blockIdx.y * p.J * p.I;
#pragma unroll
      for (int b = 0; b < 4; b++)
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int g = 0; g < 4; g++) {
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; e++) v[e] = acc[a][b][g * 4 + e];
            *reinterpret_cast<f32x4*>(out + (int64_t)(jw + b * 32) * p.I + iw + a * 32 + g * 8) = v;
          }
    } else {
#pragma unroll
      for (int b = 0; b < 4; b++)
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int g = 0; g < 4; g++) {
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; e++) v[e] = (bf16_t)acc[a][b][g * 4 + e];
            *reinterpret_cast<bf16x4*>(p.C + (int64_t)(jw + b * 32) * p.I + iw + a * 32 + g * 8) = v;
          }
    }
  } else {
    // Z = acc + bias, rounded to bf16 and stored; A = GELU(stored Z); per output row j, mean and sum of squared
    // deviations of A over this wave's 128 columns: 64 values in the lane, 64 in lane ^ 32.
    f32x4 bias4[4][4];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int g = 0; g < 4; g++) bias4[a][g] = *reinterpret_cast<const f32x4*>(p.bias + iw + a * 32 + g * 8);
    const int stat_tile = (i0 + wi * 128) >> 7;
#pragma unroll
    for (int b = 0; b < 4; b++) {
      const int64_t j = jw + b * 32;
      float sum = 0.0f;
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
          bf16x4 zs;
#pragma unroll
          for (int e = 0; e < 4; e++) {
            zs[e] = (bf16_t)(acc[a][b][g * 4 + e] + bias4[a][g][e]);
            const float act = gelu<float>((float)zs[e]);
            acc[a][b][g * 4 + e] = act;
            sum += act;
          }
          *reinterpret_cast<bf16x4*>(p.C + j * p.I + iw + a * 32 + g * 8) = zs;
        }
      sum += __shfl_xor(sum, 32, kWave);
      const float mean = sum * (1.0f / 128.0f);
      float m2 = 0.0f;
#pragma unroll
      for (int a = 0; a < 4; a++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const float d = acc[a][b][r] - mean;
          m2 = __builtin_fmaf(d, d, m2);
        }
      m2 += __shfl_xor(m2, 32, kWave);
      if (half == 0) {
        f32x2 o; o[0] = mean; o[1] = m2;
        p.part[(int64_t)stat_tile * p.J + j] = o;
      }
    }
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

template <bool P_RM, bool Q_RM, int EPI> void launch(const FastParams& p, hipStream_t s) {
  static bool configured = false;   // raise the dynamic LDS limit once per kernel
  auto kern = gemm_bf16_kernel<P_RM, Q_RM, EPI>;
  if (!configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    configured = true;
  }
  const dim3 grid((unsigned)(p.tiles_i * p.tiles_j), (unsigned)p.split);
  hipLaunchKernelGGL(kern, grid, dim3(256), kLdsBytes, s, p);
}

bool dims_ok(int64_t I, int64_t J, int64_t R) {
  return I > 0 && J > 0 && R > 0 && I % kTile == 0 && J % kTile == 0 && R % kBK == 0 &&
         I <= (1 << 24) && J <= (1 << 24) && (I / kTile) * (J / kTile) <= (1 << 30);
}

}  // namespace

bool fast_f1_supported(int64_t M, int64_t K, int64_t N) { return dims_ok(N, M, K); }
bool fast_b3_supported(int64_t M, int64_t K, int64_t N) { return dims_ok(K, M, N); }
bool fast_b4_supported(int64_t M, int64_t K, int64_t N) { return dims_ok(K, N, M); }
int fast_f1_stat_tile_w() { return 128; }

void launch_fast_f1(int64_t M, int64_t K, int64_t N, const void* X, const void* W, const float* bias, void* Zsave,
                    void* part, hipStream_t s) {
  FastParams p = {};
  p.P = (const bf16_t*)W; p.Q = (const bf16_t*)X; p.ldp = K; p.ldq = K;
  p.C = (bf16_t*)Zsave; p.bias = bias; p.part = (f32x2*)part;
  p.I = (int)N; p.J = (int)M; p.tiles_i = (int)(N / kTile); p.tiles_j = (int)(M / kTile);
  p.nkt = (int)(K / kBK); p.split = 1;
  launch<false, false, EPI_F1>(p, s);
}

void launch_fast_b3(int64_t M, int64_t K, int64_t N, const void* dZ, const void* W, void* dX, hipStream_t s) {
  FastParams p = {};
  p.P = (const bf16_t*)W; p.Q = (const bf16_t*)dZ; p.ldp = K; p.ldq = N;
  p.C = (bf16_t*)dX;
  p.I = (int)K; p.J = (int)M; p.tiles_i = (int)(K / kTile); p.tiles_j = (int)(M / kTile);
  p.nkt = (int)(N / kBK); p.split = 1;
  launch<true, false, EPI_STORE>(p, s);
}

// Split of the reduction over M so that small dW outputs still fill the chip: each part keeps >= 8 slices.
int fast_b4_split(int64_t M, int64_t K, int64_t N) {
  const int64_t tiles = (K / kTile) * (N / kTile);
  const int64_t slices = M / kBK;
  int split = 1;
  while (tiles * split * 2 <= 256 && slices % (split * 2) == 0 && slices / (split * 2) >= 8) split *= 2;
  return split;
}

void launch_fast_b4(int64_t M, int64_t K, int64_t N, int split, const void* dZ, const void* X, void* dW, void* dwpart,
                    hipStream_t s) {
  FastParams p = {};
  p.P = (const bf16_t*)X; p.Q = (const bf16_t*)dZ; p.ldp = K; p.ldq = N;
  p.C = (bf16_t*)dW; p.Cpart = (float*)dwpart;
  p.I = (int)K; p.J = (int)N; p.tiles_i = (int)(K / kTile); p.tiles_j = (int)(N / kTile);
  p.nkt = (int)(M / kBK / split); p.split = split;
  launch<true, true, EPI_STORE>(p, s);
  if (split > 1) {
    const int64_t n = N * K;
    hipLaunchKernelGGL(reduce_split_kernel, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, s,
                       (const float*)dwpart, split, n, (bf16_t*)dW);
  }
}

}  // namespace fdl
