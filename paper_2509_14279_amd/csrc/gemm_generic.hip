// Generic MFMA GEMM for the fused dense-layer block: any shape, any alignment, both storage types.
//
//     C[i][j] = sum_r A(i,r) * B(j,r)          I x J outputs, reduction length R
//
// Used for all three contractions of the block when the tuned bf16 kernel does not apply:
//   F1  Z  = X W^T + b   A = X  (r = k contiguous)   B = W  (r = k contiguous)
//   B3  dX = dZ W        A = dZ (r = n contiguous)   B = W  (r = n is the row index)
//   B4  dW = dZ^T X      A = dZ (r = m is the row index)   B = X (r = m is the row index)
// (the three linear-layer products of the paper's linear forward/backward tasks, appendix
// "Highlighted CUDA Kernels: Code", done here on the matrix cores instead of one thread or warp per
// output element).
//
// Storage fp32  -> operands widened to fp64 in registers, v_mfma_f64_16x16x4_f64, fp64 accumulators.
// Storage bf16  -> operands widened to fp32 at the global load (one LDS layout for both storage types), packed back
//                  to bf16 at the fragment (exact), v_mfma_f32_16x16x16_bf16, fp32 accumulators.
// A lane's fragment is the four reduction indices 4*(lane/16)+s, s = 0..3, of a 16-deep slice for A and B alike
// (row/col = lane%16): four steps of the fp64 instruction, which takes one value per lane and step, or the
// operand of one bf16 instruction; an r-contiguous operand is read from LDS with one 16-byte read per fragment.
//
// Workgroup: 256 threads = 4 waves as 2x2; wave tile (16*WB)^2; block tile (32*WB)^2; 16-deep reduction
// slices, double-buffered in LDS with the global loads of the next two slices in flight during the MFMAs.
#include "common.hip.h"
#include "internal.h"

namespace fdl {
namespace {

// EPI_STORE: C = acc (+ bias[j] when given).  EPI_F1: bias, GELU and partial row statistics.  EPI_STORE_F32: fp32 C.
// EPI_RELU: C = max(acc + bias[j], 0).  EPI_MASK: C = aux[i][j] where acc + bias[j] > 0, else 0.
enum { EPI_STORE = 0, EPI_F1 = 1, EPI_STORE_F32 = 2, EPI_RELU = 3, EPI_MASK = 4 };

struct GemmParams {
  const void* A; const void* B; void* C;
  const float* bias; f32x2* part;
  const void* aux;       // [I][J] in the storage type (EPI_MASK)
  int64_t I, J, R, lda, ldb;
  int a_vec, b_vec;
  int wide;              // both contiguous extents hold at least one chunk of four: ragged rows take vector loads too
};

template <class AccT> struct Mma;
// fp64: v_mfma_f64_16x16x4_f64.  (Four v_mfma_f64_4x4x4_4b with the B fragment rotated by blocks of four lanes
// compute the same product; over the chip that form sustains 70 TFLOP/s against 77 for this one, measured with the
// accumulators held in AGPRs, and in this kernel it ran 20 % slower.)
template <> struct Mma<double> {
  typedef f64x4 acc_t;
  static constexpr int kRowsPerLane = 4;      // distinct output rows among a lane's four accumulator elements
  static constexpr int kRowLanes = 16;        // lanes that share a row
  static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64((double)a, (double)b, c, 0, 0, 0);
  }
  // the lane's four reduction steps of a 16-deep slice
  static __device__ __forceinline__ acc_t mma4(const float (&a)[4], const float (&b)[4], acc_t c) {
#pragma unroll
    for (int s = 0; s < 4; s++) c = mma(a[s], b[s], c);
    return c;
  }
  // accumulator register r of lane l holds output row 4r + l/16, column l%16
  static __device__ __forceinline__ int row(int lane, int r) { return r * 4 + (lane >> 4); }
  static __device__ __forceinline__ int col(int lane, int) { return lane & 15; }
};
template <> struct Mma<float> {
  typedef f32x4 acc_t;
  static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
  // The values are bf16 numbers widened to fp32 on their way through LDS, so packing the lane's four reduction
  // steps back into bf16 is exact and one v_mfma_f32_16x16x16_bf16 (k = 4 (lane/16) + e, the same assignment of
  // reduction indices to lanes) does the work of four fp32 steps at sixteen times the rate.
  static __device__ __forceinline__ acc_t mma4(const float (&a)[4], const float (&b)[4], acc_t c) {
    typedef __attribute__((ext_vector_type(4))) short s16x4;
    bf16x4 pa, pb;
#pragma unroll
    for (int s = 0; s < 4; s++) { pa[s] = (bf16_t)a[s]; pb[s] = (bf16_t)b[s]; }
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, pa), __builtin_bit_cast(s16x4, pb), c, 0, 0, 0);
  }
  // accumulator register r of lane l holds output row 4(l/16) + r, column l%16
  static constexpr int kRowsPerLane = 4;
  static constexpr int kRowLanes = 16;
  static __device__ __forceinline__ int row(int lane, int r) { return (lane >> 4) * 4 + r; }
  static __device__ __forceinline__ int col(int lane, int) { return lane & 15; }
};

template <class T> __device__ __forceinline__ void load4(const T* p, float (&v)[4]);
template <> __device__ __forceinline__ void load4<float>(const float* p, float (&v)[4]) {
  const f32x4 t = *reinterpret_cast<const f32x4*>(p);
  v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
}
template <> __device__ __forceinline__ void load4<bf16_t>(const bf16_t* p, float (&v)[4]) {
  const bf16x4 t = *reinterpret_cast<const bf16x4*>(p);
  v[0] = (float)t[0]; v[1] = (float)t[1]; v[2] = (float)t[2]; v[3] = (float)t[3];
}

// the same from an address that is only element-aligned (rows of a ragged matrix start anywhere): the compiler picks
// the widest load the target allows for the stated alignment
template <class T> __device__ __forceinline__ void load4u(const T* p, float (&v)[4]);
template <> __device__ __forceinline__ void load4u<float>(const float* p, float (&v)[4]) {
  typedef float f32x4_u __attribute__((ext_vector_type(4), aligned(4)));
  const f32x4_u t = *reinterpret_cast<const f32x4_u*>(p);
  v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
}
template <> __device__ __forceinline__ void load4u<bf16_t>(const bf16_t* p, float (&v)[4]) {
  typedef __bf16 bf16x4_u __attribute__((ext_vector_type(4), aligned(2)));
  const bf16x4_u t = *reinterpret_cast<const bf16x4_u*>(p);
  v[0] = (float)t[0]; v[1] = (float)t[1]; v[2] = (float)t[2]; v[3] = (float)t[3];
}

// One operand's BT x 16 slice: global -> registers -> LDS, and LDS -> MFMA fragments.
// RC  (reduction-contiguous in memory): LDS layout [BT][20] floats (16 + 4 pad: 16-byte accesses of 8
//      consecutive rows fall on 8 disjoint groups of 4 banks).
// !RC (row index is the reduction index): LDS layout [16][BT+4] floats.
enum { kElements = 0, kVecAligned = 1, kVecAnywhere = 2 };   // how an operand's chunks of four elements are loaded
template <class T, bool RC, int BT> struct Operand {
  static constexpr int kChunks = BT * 16 / 4;
  static constexpr int kPerThread = kChunks / 256;
  static constexpr int kFloats = BT * 20;
  static_assert(kPerThread >= 1, "block tile too small for 256 threads");

  // Loads never depend on a per-lane condition: an element outside the matrix is read from the nearest row and
  // column inside it (always valid memory) and replaced by zero when the slice goes to LDS.  A load under a
  // per-lane branch, or one merged with a zero in its destination register, would make the wavefront wait for
  // every load in flight first, which serialises the slices' trips to memory.
  // mode kVecAligned: 16-byte (fp32) or 8-byte (bf16) loads - base and pitch aligned and the contiguous extent a
  //   multiple of 4, so a chunk is inside the matrix entirely or not at all.
  // mode kVecAnywhere: the same loads from element-aligned addresses (ragged pitch); a chunk that straddles the end
  //   of its row is read from the last four elements of the row instead and shifted back when it is stashed.
  // mode kElements: one load per element (a contiguous extent below 4).
  static __device__ __forceinline__ void fetch(const T* base, int64_t ld, int64_t i0, int64_t I, int64_t r0, int64_t R,
                                               int mode, int tid, float (&reg)[kPerThread][4]) {
#pragma unroll
    for (int q = 0; q < kPerThread; q++) {
      const int c = tid + q * 256;
      // (row, first column) of the chunk in memory: RC rows are tile rows, !RC rows are reduction indices
      const int64_t row = RC ? i0 + (c >> 2) : r0 + c / (BT / 4);
      const int64_t col = RC ? r0 + (c & 3) * 4 : i0 + (c % (BT / 4)) * 4;
      const int64_t rows = RC ? I : R, cols = RC ? R : I;
      const T* prow = base + (row < rows ? row : rows - 1) * ld;
      if (mode == kVecAligned) {
        load4<T>(prow + (col + 3 < cols ? col : cols - 4), reg[q]);
      } else if (mode == kVecAnywhere) {
        load4u<T>(prow + (col + 3 < cols ? col : cols - 4), reg[q]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; e++) reg[q][e] = to_f32<T>(prow[col + e < cols ? col + e : cols - 1]);
      }
    }
  }

  // r0: first reduction index of the slice that `reg` holds
  static __device__ __forceinline__ void stash(float* lds, int tid, int64_t i0, int64_t I, int64_t r0, int64_t R,
                                               int mode, const float (&reg)[kPerThread][4]) {
#pragma unroll
    for (int q = 0; q < kPerThread; q++) {
      const int c = tid + q * 256;
      const int64_t row = RC ? i0 + (c >> 2) : r0 + c / (BT / 4);
      const int64_t col = RC ? r0 + (c & 3) * 4 : i0 + (c % (BT / 4)) * 4;
      const int64_t rows = RC ? I : R, cols = RC ? R : I;
      // kVecAnywhere: the chunk was read `shift` elements early where it straddles the end of the row
      const int shift = (mode == kVecAnywhere && col + 3 >= cols) ? (int)(col - (cols - 4)) : 0;
      f32x4 t;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        float v = reg[q][e];
        if (mode == kVecAnywhere) {
#pragma unroll
          for (int h = 1; e + h < 4; h++) v = shift == h ? reg[q][e + h] : v;
        }
        t[e] = (row < rows && col + e < cols) ? v : 0.0f;
      }
      if (RC) {
        *reinterpret_cast<f32x4*>(lds + (c >> 2) * 20 + (c & 3) * 4) = t;
      } else {
        *reinterpret_cast<f32x4*>(lds + (c / (BT / 4)) * (BT + 4) + (c % (BT / 4)) * 4) = t;
      }
    }
  }

  // fragment for tile row `row` (within the block tile): the 4 reduction indices 4g..4g+3, g = lane/16
  static __device__ __forceinline__ void frag(const float* lds, int row, int g, float (&f)[4]) {
    if (RC) {
      const f32x4 t = *reinterpret_cast<const f32x4*>(lds + row * 20 + g * 4);
      f[0] = t[0]; f[1] = t[1]; f[2] = t[2]; f[3] = t[3];
    } else {
#pragma unroll
      for (int s = 0; s < 4; s++) f[s] = lds[(g * 4 + s) * (BT + 4) + row];
    }
  }
};

// The reduction loop of one block tile.  Global loads run kDepth - 1 slices ahead of the MFMAs in a ring of register
// sets (slice k lives in set k % kDepth): a 16-deep slice is only a few hundred nanoseconds of matrix work, less than
// a trip to memory, and shapes with few tiles per compute unit have no other wavefronts to hide it behind.  LDS stays
// double-buffered.  The body has no branches: past the last slice the loop re-fetches and re-stashes the last slice
// (into the LDS buffer that is not read again) instead of testing, so that the compiler can count the loads in flight
// exactly and wait only for the oldest.  MODE: how both operands are loaded (see Operand; a compile-time property of
// the loop for the same reason).
template <class T, class AccT, bool A_RC, bool B_RC, int WB, int MODE>
__device__ __forceinline__ void generic_mainloop(const GemmParams& p, int64_t i0, int64_t j0, float (*lds)[2][32 * WB * 20],
                                                 typename Mma<AccT>::acc_t (&acc)[WB][WB]) {
  constexpr int BT = 32 * WB;
  typedef Operand<T, A_RC, BT> OpA;
  typedef Operand<T, B_RC, BT> OpB;
  constexpr int kDepth = 3;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int g = lane >> 4, l16 = lane & 15;
  const T* A = static_cast<const T*>(p.A);
  const T* B = static_cast<const T*>(p.B);
  float ra[kDepth][OpA::kPerThread][4], rb[kDepth][OpB::kPerThread][4];
  const int64_t slices = (p.R + 15) / 16, last = slices - 1;
#pragma unroll
  for (int d = 0; d < kDepth - 1; d++) {
    const int64_t r0 = (d < last ? d : last) * 16;
    OpA::fetch(A, p.lda, i0, p.I, r0, p.R, MODE, tid, ra[d]);
    OpB::fetch(B, p.ldb, j0, p.J, r0, p.R, MODE, tid, rb[d]);
  }
  OpA::stash(lds[0][0], tid, i0, p.I, 0, p.R, MODE, ra[0]);
  OpB::stash(lds[0][1], tid, j0, p.J, 0, p.R, MODE, rb[0]);
  __syncthreads();

  auto step = [&](int64_t kt, int d) __attribute__((always_inline)) {
    const int cur = (int)(kt & 1);
    const int64_t rf = (kt + kDepth - 1 < last ? kt + kDepth - 1 : last) * 16;
    OpA::fetch(A, p.lda, i0, p.I, rf, p.R, MODE, tid, ra[(d + kDepth - 1) % kDepth]);
    OpB::fetch(B, p.ldb, j0, p.J, rf, p.R, MODE, tid, rb[(d + kDepth - 1) % kDepth]);
    float fa[WB][4], fb[WB][4];
#pragma unroll
    for (int a = 0; a < WB; a++) OpA::frag(lds[cur][0], wi * 16 * WB + a * 16 + l16, g, fa[a]);
#pragma unroll
    for (int b = 0; b < WB; b++) OpB::frag(lds[cur][1], wj * 16 * WB + b * 16 + l16, g, fb[b]);
#pragma unroll
    for (int a = 0; a < WB; a++)
#pragma unroll
      for (int b = 0; b < WB; b++) acc[a][b] = Mma<AccT>::mma4(fa[a], fb[b], acc[a][b]);
    // the accumulators stay in AGPRs between slices (left to itself the compiler moves them to VGPRs and back once
    // per trip through the unrolled loop)
#pragma unroll
    for (int a = 0; a < WB; a++)
#pragma unroll
      for (int b = 0; b < WB; b++) asm volatile("" : "+a"(acc[a][b]));
    const int64_t rs = (kt + 1 < last ? kt + 1 : last) * 16;
    OpA::stash(lds[cur ^ 1][0], tid, i0, p.I, rs, p.R, MODE, ra[(d + 1) % kDepth]);
    OpB::stash(lds[cur ^ 1][1], tid, j0, p.J, rs, p.R, MODE, rb[(d + 1) % kDepth]);
    __syncthreads();
  };
#pragma unroll
  for (int a = 0; a < WB; a++)
#pragma unroll
    for (int b = 0; b < WB; b++) asm volatile("" : "+a"(acc[a][b]));
  int64_t k0 = 0;
  for (; k0 + kDepth <= slices; k0 += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; d++) step(k0 + d, d);
  }
#pragma unroll
  for (int d = 0; d < kDepth - 1; d++)
    if (k0 + d < slices) step(k0 + d, d);   // uniform over the workgroup
}

template <class T, class AccT, bool A_RC, bool B_RC, int WB, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmParams p) {
  constexpr int BT = 32 * WB;
  typedef typename Mma<AccT>::acc_t acc_t;
  __shared__ __attribute__((aligned(16))) float lds[2][2][BT * 20];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave >> 1, wj = wave & 1;
  const int64_t tiles_j = (p.J + BT - 1) / BT;
  const int64_t i0 = (int64_t)(blockIdx.x / tiles_j) * BT, j0 = (int64_t)(blockIdx.x % tiles_j) * BT;

  acc_t acc[WB][WB];
#pragma unroll
  for (int a = 0; a < WB; a++)
#pragma unroll
    for (int b = 0; b < WB; b++)
#pragma unroll
      for (int r = 0; r < 4; r++) acc[a][b][r] = 0;

  if (p.a_vec && p.b_vec) generic_mainloop<T, AccT, A_RC, B_RC, WB, kVecAligned>(p, i0, j0, lds, acc);
  else if (p.wide) generic_mainloop<T, AccT, A_RC, B_RC, WB, kVecAnywhere>(p, i0, j0, lds, acc);
  else generic_mainloop<T, AccT, A_RC, B_RC, WB, kElements>(p, i0, j0, lds, acc);

  // ------------------------------------------------------------------ epilogue
  // accumulator element r of block (a, b): output row iw + 16 a + row(lane, r), column jw + 16 b + col(lane, r)
  typedef Mma<AccT> M;
  const int64_t iw = i0 + wi * 16 * WB, jw = j0 + wj * 16 * WB;
  T* C = static_cast<T*>(p.C);
  if (EPI == EPI_STORE_F32) {
    float* Cf = static_cast<float*>(p.C);
#pragma unroll
    for (int a = 0; a < WB; a++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int64_t i = iw + a * 16 + M::row(lane, r);
#pragma unroll
        for (int b = 0; b < WB; b++) {
          const int64_t j = jw + b * 16 + M::col(lane, r);
          if (i < p.I && j < p.J) Cf[i * p.J + j] = (float)acc[a][b][r];
        }
      }
  } else if (EPI == EPI_STORE || EPI == EPI_RELU || EPI == EPI_MASK) {
    AccT bias[WB][4];
#pragma unroll
    for (int b = 0; b < WB; b++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int64_t j = jw + b * 16 + M::col(lane, r);
        bias[b][r] = (p.bias != nullptr && j < p.J) ? (AccT)p.bias[j] : (AccT)0;
      }
    const T* aux = static_cast<const T*>(p.aux);
#pragma unroll
    for (int a = 0; a < WB; a++)
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int64_t i = iw + a * 16 + M::row(lane, r);
#pragma unroll
        for (int b = 0; b < WB; b++) {
          const int64_t j = jw + b * 16 + M::col(lane, r);
          if (i < p.I && j < p.J) {
            const AccT z = acc[a][b][r] + bias[b][r];
            if (EPI == EPI_MASK) C[i * p.J + j] = z > (AccT)0 ? aux[i * p.J + j] : (T)0.0f;
            else if (EPI == EPI_RELU) C[i * p.J + j] = to_storage<T, AccT>(z > (AccT)0 ? z : (AccT)0);
            else C[i * p.J + j] = to_storage<T, AccT>(z);
          }
        }
      }
  } else {
    // Z = acc + bias, stored rounded; A = GELU(stored Z); two-pass mean / sum of squared deviations over
    // this wave's 16*WB columns of the row, reduced across the lanes that share the row (written for any
    // assignment of a lane's accumulator elements to rows: kRowsPerLane of them, kRowLanes lanes per row).
    constexpr int RPL = M::kRowsPerLane;
    constexpr int NE = (4 / RPL) * WB;           // elements of one row held by a lane
    const int64_t tile = jw / (16 * WB);
    int64_t nvalid = p.J - jw;
    if (nvalid > 16 * WB) nvalid = 16 * WB;
#pragma unroll
    for (int a = 0; a < WB; a++)
#pragma unroll
      for (int slot = 0; slot < RPL; slot++) {
        const int64_t i = iw + a * 16 + M::row(lane, slot);
        AccT act[NE];
        bool ok[NE];
        AccT sum = 0;
        int n = 0;
#pragma unroll
        for (int b = 0; b < WB; b++)
#pragma unroll
          for (int r = 0; r < 4; r++) {
            if (RPL == 4 && r != slot) continue;
            const int64_t j = jw + b * 16 + M::col(lane, r);
            ok[n] = j < p.J;
            const AccT bias = ok[n] ? (AccT)p.bias[j] : (AccT)0;
            const T zs = to_storage<T, AccT>(acc[a][b][r] + bias);
            if (ok[n] && i < p.I) C[i * p.J + j] = zs;
            act[n] = ok[n] ? gelu<AccT>((AccT)to_f32<T>(zs)) : (AccT)0;
            sum += act[n];
            n++;
          }
#pragma unroll
        for (int m = 1; m < M::kRowLanes; m <<= 1) sum += __shfl_xor(sum, m, kWave);
        const AccT mean = nvalid > 0 ? sum / (AccT)nvalid : (AccT)0;
        AccT m2 = 0;
#pragma unroll
        for (int e = 0; e < NE; e++) {
          const AccT d = act[e] - mean;
          m2 += ok[e] ? d * d : (AccT)0;
        }
#pragma unroll
        for (int m = 1; m < M::kRowLanes; m <<= 1) m2 += __shfl_xor(m2, m, kWave);
        if ((lane & (M::kRowLanes - 1)) == 0 && i < p.I && nvalid > 0) {
          f32x2 o; o[0] = (float)mean; o[1] = (float)m2;
          p.part[tile * p.I + i] = o;
        }
      }
  }
}

template <class T, bool A_RC, bool B_RC, int WB, int EPI>
void launch_one(const GemmParams& p, hipStream_t s) {
  typedef typename ComputeOf<T>::type AccT;
  constexpr int BT = 32 * WB;
  const int64_t tiles = ((p.I + BT - 1) / BT) * ((p.J + BT - 1) / BT);
  hipLaunchKernelGGL((gemm_generic_kernel<T, AccT, A_RC, B_RC, WB, EPI>), dim3((unsigned)tiles), dim3(256), 0, s, p);
}

// Vector loads need an aligned base, a pitch that keeps every 4-element chunk aligned, and a contiguous extent that is
// a whole number of chunks (a chunk is then inside the matrix entirely or not at all).
void set_vec(GemmParams* p, const GemmDesc& g, bool a_rc, bool b_rc, size_t elem_bytes) {
  const size_t chunk_bytes = 4 * elem_bytes;
  const int64_t a_extent = a_rc ? g.R : g.I, b_extent = b_rc ? g.R : g.J;
  p->a_vec = ((uintptr_t)g.A % chunk_bytes == 0) && (g.lda % 4 == 0) && (a_extent % 4 == 0);
  p->b_vec = ((uintptr_t)g.B % chunk_bytes == 0) && (g.ldb % 4 == 0) && (b_extent % 4 == 0);
  p->wide = a_extent >= 4 && b_extent >= 4;
}

template <class T, int EPI> void dispatch(const GemmDesc& g, GemmParams p, hipStream_t s) {
  set_vec(&p, g, g.a_rc, g.b_rc, sizeof(T));
  const bool big = g.wb == 4;
  if (EPI == EPI_F1) {           // F1 always has both operands reduction-contiguous
    if (big) launch_one<T, true, true, 4, EPI>(p, s); else launch_one<T, true, true, 2, EPI>(p, s);
    return;
  }
  if (g.a_rc && !g.b_rc) {
    if (big) launch_one<T, true, false, 4, EPI>(p, s); else launch_one<T, true, false, 2, EPI>(p, s);
  } else if (!g.a_rc && !g.b_rc) {
    if (big) launch_one<T, false, false, 4, EPI>(p, s); else launch_one<T, false, false, 2, EPI>(p, s);
  } else if (g.a_rc && g.b_rc) {
    if (big) launch_one<T, true, true, 4, EPI>(p, s); else launch_one<T, true, true, 2, EPI>(p, s);
  } else {
    if (big) launch_one<T, false, true, 4, EPI>(p, s); else launch_one<T, false, true, 2, EPI>(p, s);
  }
}

GemmParams base_params(const GemmDesc& g) {
  GemmParams p;
  p.A = g.A; p.B = g.B; p.C = nullptr; p.bias = nullptr; p.part = nullptr; p.aux = nullptr;
  p.I = g.I; p.J = g.J; p.R = g.R; p.lda = g.lda; p.ldb = g.ldb; p.a_vec = 0; p.b_vec = 0; p.wide = 0;
  return p;
}

}  // namespace

void launch_generic_f1(int dt, const GemmDesc& g, const float* bias, void* Zsave, void* part, hipStream_t s) {
  GemmParams p = base_params(g);
  p.C = Zsave; p.bias = bias; p.part = static_cast<f32x2*>(part);
  if (dt == kF32) dispatch<float, EPI_F1>(g, p, s); else dispatch<bf16_t, EPI_F1>(g, p, s);
}

// only the operand orientation of the dW contraction (both operands indexed by the reduction row) is needed
void launch_generic_store_f32(const GemmDesc& g, float* C, hipStream_t s) {
  GemmParams p = base_params(g);
  p.C = C;
  set_vec(&p, g, false, false, 2);
  if (g.wb == 4) launch_one<bf16_t, false, false, 4, EPI_STORE_F32>(p, s);
  else launch_one<bf16_t, false, false, 2, EPI_STORE_F32>(p, s);
}

// C[i][j] = f(sum_r A(i,r) B(j,r) + bias[j]), both operands reduction-contiguous (the forward product's orientation):
// kind 0 plain (bias may be null), 1 max(., 0), 2 aux[i][j] where the sum is positive else 0
void launch_generic_xwt(int dt, int kind, const GemmDesc& g, const float* bias, const void* aux, void* C, hipStream_t s) {
  GemmParams p = base_params(g);
  p.C = C; p.bias = bias; p.aux = aux;
  set_vec(&p, g, true, true, dt == kF32 ? 4 : 2);
  const bool big = g.wb == 4;
#define FDL_GX(T, EPI) do { if (big) launch_one<T, true, true, 4, EPI>(p, s); else launch_one<T, true, true, 2, EPI>(p, s); } while (0)
  if (dt == kF32) {
    if (kind == 1) FDL_GX(float, EPI_RELU); else if (kind == 2) FDL_GX(float, EPI_MASK); else FDL_GX(float, EPI_STORE);
  } else {
    if (kind == 1) FDL_GX(bf16_t, EPI_RELU); else if (kind == 2) FDL_GX(bf16_t, EPI_MASK); else FDL_GX(bf16_t, EPI_STORE);
  }
#undef FDL_GX
}

void launch_generic_store(int dt, const GemmDesc& g, void* C, hipStream_t s) {
  GemmParams p = base_params(g);
  p.C = C;
  if (dt == kF32) dispatch<float, EPI_STORE>(g, p, s); else dispatch<bf16_t, EPI_STORE>(g, p, s);
}

}  // namespace fdl
