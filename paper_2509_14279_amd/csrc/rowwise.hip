// Streaming (HBM-bound) phases of the fused dense-layer block: LayerNorm statistics merge and
// normalisation (forward), the LayerNorm/GELU gradient row pass with its column partial sums
// (backward), and the column reduction that finishes dbeta, dgamma, db.
//
// Row reductions follow the idiom of the paper's row-normalisation kernels (appendix "Highlighted CUDA
// Kernels", LayerNorm forward and Llama RMSNorm forward: vector loads, wavefront shuffles, a small LDS
// exchange between wavefronts) with 64-wide wavefronts; the bias-style column sums are laid out so that
// consecutive lanes read consecutive columns (the paper's linear backward bias kernel walks a column with
// stride N instead).
//
// Arithmetic type C is one level above the storage type T: fp64 for fp32 storage, fp32 for bf16 storage.
#include "common.hip.h"
#include "internal.h"

namespace fdl {
namespace {

// ------------------------------------------------------------------------------------------------
// FS: merge per-(row, column tile) partial (mean, sum of squared deviations) pairs with the pairwise
// update of Chan et al., in fp64.  part is [tiles][M].  Sixteen lanes share a row: lane l merges tiles l, l + 16, ...
// in order, then the sixteen (count, mean, M2) triples are merged pairwise across the lanes - the update is
// associative, and with one thread per row a matrix of a few thousand rows kept a dozen workgroups busy with a
// serial chain of fp64 divisions per tile.
struct Moments { double n, mu, m2; };
__device__ __forceinline__ Moments merge_moments(const Moments& a, const Moments& b) {
  Moments r;
  r.n = a.n + b.n;
  const double d = b.mu - a.mu, w = r.n > 0.0 ? b.n / r.n : 0.0;
  r.mu = a.mu + d * w;
  r.m2 = a.m2 + b.m2 + d * d * a.n * w;
  return r;
}
__global__ __launch_bounds__(256) void stats_finalize_kernel(const f32x2* __restrict__ part, int tiles, int tile_w,
                                                             int64_t M, int64_t N, float eps,
                                                             float* __restrict__ mean, float* __restrict__ rstd) {
  constexpr int kLanes = 16;
  const int l = threadIdx.x & (kLanes - 1);
  const int64_t m = (int64_t)blockIdx.x * (256 / kLanes) + (threadIdx.x / kLanes);
  const int64_t mc = m < M ? m : M - 1;      // lanes past the last row redo it (no early exit before the shuffles)
  Moments acc = {0.0, 0.0, 0.0};
  for (int t = l; t < tiles; t += kLanes) {
    int64_t nb = N - (int64_t)t * tile_w;
    if (nb <= 0) break;
    if (nb > tile_w) nb = tile_w;
    const f32x2 p = part[(int64_t)t * M + mc];
    const Moments x = {(double)nb, (double)p[0], (double)p[1]};
    acc = merge_moments(acc, x);
  }
#pragma unroll
  for (int k = 1; k < kLanes; k <<= 1) {
    Moments o;
    o.n = __shfl_xor(acc.n, k, kWave); o.mu = __shfl_xor(acc.mu, k, kWave); o.m2 = __shfl_xor(acc.m2, k, kWave);
    // both lanes of a pair merge the same two triples in the same order (lower lane's first)
    acc = (l & k) ? merge_moments(o, acc) : merge_moments(acc, o);
  }
  if (l == 0 && m < M) {
    mean[m] = (float)acc.mu;
    rstd[m] = (float)(1.0 / sqrt(acc.m2 / (double)N + (double)eps));
  }
}

// ------------------------------------------------------------------------------------------------
// F2: Y = (GELU(Zsave) - mean) * rstd * gamma + beta.  A workgroup owns a strip of 256*V columns and a
// block of rows; gamma and beta for the thread's V columns stay in registers across the rows.
template <class T, int V>
// (Z and Y may be the same buffer - the forward-only entry point normalises in place; each element is read by the
// thread that writes it, before it writes it - so the two are not declared restrict.)
__global__ __launch_bounds__(256) void f2_kernel(int64_t M, int64_t N, int rows_per_wg, int strips,
                                                 const T* Z, const float* __restrict__ mean,
                                                 const float* __restrict__ rstd, const float* __restrict__ gamma,
                                                 const float* __restrict__ beta, T* Y) {
  typedef typename ComputeOf<T>::type C;
  const int strip = blockIdx.x % strips;
  const int64_t rb = blockIdx.x / strips;
  const int64_t col = ((int64_t)strip * 256 + threadIdx.x) * V;
  if (col >= N) return;
  C gm[V], bt[V];
#pragma unroll
  for (int v = 0; v < V; v++) { gm[v] = (C)gamma[col + v]; bt[v] = (C)beta[col + v]; }
  const int64_t r0 = rb * rows_per_wg;
  int64_t r1 = r0 + rows_per_wg;
  if (r1 > M) r1 = M;
#pragma unroll 4
  for (int64_t r = r0; r < r1; r++) {
    C z[V], y[V];
    VecIO<T, V>::load(Z + r * N + col, z);
    const C mu = (C)mean[r], rs = (C)rstd[r];
#pragma unroll
    for (int v = 0; v < V; v++) y[v] = (gelu<C>(z[v]) - mu) * rs * gm[v] + bt[v];
    VecIO<T, V>::store(Y + r * N + col, y);
  }
}

// ------------------------------------------------------------------------------------------------
// F2 with its own statistics (bf16 storage, N % 8 == 0, N <= 512 CH): a wavefront owns a row and keeps it in
// registers over three sweeps (GELU and sum; deviations and their squares; scale, shift, store), so Zsave is read
// once, no partial statistics pass through memory and no barrier separates the sweeps.  Lane l holds the 8-element
// vectors c*64 + l, c < CH, of its row (every load and store of a wavefront covers 1 KB of one row); the next
// row's vectors are fetched while the current row is processed.  gamma and beta sit in LDS, permuted so that a
// lane's four 16-byte reads per vector are lane-contiguous.  Workgroups of NT/64 wavefronts walk the rows with
// stride (8 wavefronts; 4 for the widest masked variant, whose extra per-vector state needs the larger register
// budget of one wavefront per SIMD).
// FULL: N == 512 CH, every lane holds every vector.  Otherwise the vectors past the end of the row are fetched
// from a clamped address, masked to zero (GELU(0) = 0 adds nothing to the sum), left out of the squared
// deviations and never stored; the code stays free of divergent branches either way.
// ACT selects what is normalised: ACT_GELU the GELU of the input (the block's second forward phase; Z and Y may then
// be the same buffer - a lane reads its part of a row before it writes it - so they are not declared restrict),
// ACT_NONE the input itself (stand-alone LayerNorm forward), ACT_RMS the input without mean subtraction and without
// beta (RMSNorm forward: y = x (mean(x^2) + eps)^-1/2 w; mean and rstd are not written).
enum { ACT_GELU = 0, ACT_NONE = 1, ACT_RMS = 2 };
template <int CH, bool FULL, int NT, int ACT>
__global__ __launch_bounds__(NT) void f2_rows_kernel(int64_t M, int64_t N, float eps, const bf16_t* Z,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      bf16_t* Y, float* __restrict__ mean,
                                                      float* __restrict__ rstd) {
  // products are formed once and reused (fusing GELU's final multiplication into each later use would keep
  // both of its factors alive for every element of the row); the fused operations wanted are written out
#pragma clang fp contract(off)
  extern __shared__ f32x4 gb[];   // [CH][4][64]: gamma[0:4], gamma[4:8], beta[0:4], beta[4:8] of vector c*64 + lane
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  typedef GaussTable<false> GT;
  typedef __attribute__((address_space(3))) float lds_float;
  float* htab = reinterpret_cast<float*>(gb + CH * 4 * 64);           // Phi - 1/2 for every bf16 magnitude
  const uint32_t horg = GT::origin((uint32_t)(uintptr_t)(const lds_float*)htab);
  if (ACT == ACT_GELU) GT::build(htab, threadIdx.x, NT);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: row addresses stay scalar
  const int nvec = (int)(N >> 3);
  for (int idx = threadIdx.x; idx < CH * 64; idx += NT) {
    const int64_t src = (int64_t)(idx < nvec ? idx : nvec - 1) * 8;
    const int c = idx >> 6, l = idx & 63;
    gb[(c * 4 + 0) * 64 + l] = *reinterpret_cast<const f32x4*>(gamma + src);
    gb[(c * 4 + 1) * 64 + l] = *reinterpret_cast<const f32x4*>(gamma + src + 4);
    if (ACT != ACT_RMS) {
      gb[(c * 4 + 2) * 64 + l] = *reinterpret_cast<const f32x4*>(beta + src);
      gb[(c * 4 + 3) * 64 + l] = *reinterpret_cast<const f32x4*>(beta + src + 4);
    }
  }
  __syncthreads();
  const int64_t nw = (int64_t)gridDim.x * (NT / 64);
  const float inv_n = 1.0f / (float)N;
  // per-lane element offset of vector c inside a row, and whether the row has that vector
  int voff[CH];
  uint32_t keep[CH];
#pragma unroll
  for (int c = 0; c < CH; c++) {
    const int vi = c * 64 + lane;
    voff[c] = (FULL || vi < nvec ? vi : nvec - 1) * 8;
    keep[c] = (FULL || vi < nvec) ? 0xffffffffu : 0u;
  }

  u32x4 raw[CH];
  // vector c of row r (past the last row: a harmless re-read of the last one, never used)
  auto fetch1 = [&](int c, const bf16_t* zr) {
    if (FULL) {
      // scalar base per vector + one shared per-lane offset (the immediate offset field reaches only 4 KB)
      const bf16_t* zc = zr + c * 512;
      asm("" : "+s"(zc));
      raw[c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(zc + lane * 8));
    } else {
      raw[c] = *reinterpret_cast<const u32x4*>(zr + voff[c]);
    }
  };
  int64_t row = (int64_t)blockIdx.x * (NT / 64) + wave;
  {
    const bf16_t* zr = Z + (row < M ? row : M - 1) * N;
#pragma unroll
    for (int c = 0; c < CH; c++) fetch1(c, zr);
  }
  for (; row < M; row += nw) {
    float a[CH][8];
    float sum = 0.0f;
    const bf16_t* znext = Z + (row + nw < M ? row + nw : M - 1) * N;
#pragma unroll
    for (int c = 0; c < CH; c++) {
#pragma unroll
      for (int h = 0; h < 4; h++) {
        const uint32_t w = FULL ? raw[c][h] : (raw[c][h] & keep[c]);
        const float z0 = __builtin_bit_cast(float, w << 16);                        // bf16 -> fp32 is a 16-bit shift
        const float z1 = __builtin_bit_cast(float, w & 0xffff0000u);
        if (ACT == ACT_GELU) {
          const float h0 = *(const lds_float*)(uintptr_t)GT::address_of(w, horg);
          const float h1 = *(const lds_float*)(uintptr_t)GT::address_of(w >> 16, horg);
          a[c][2 * h] = z0 * (0.5f + GT::with_sign_of(h0, z0));                     // GELU(z) = z Phi(z)
          a[c][2 * h + 1] = z1 * (0.5f + GT::with_sign_of(h1, z1));
        } else {
          a[c][2 * h] = z0;
          a[c][2 * h + 1] = z1;
        }
        if (ACT == ACT_RMS) {
          sum = __builtin_fmaf(z0, z0, sum);
          sum = __builtin_fmaf(z1, z1, sum);
        } else {
          sum += a[c][2 * h];
          sum += a[c][2 * h + 1];
        }
      }
      // One vector at a time (interleaving all of a row's evaluations would keep their temporaries alive), and as
      // soon as a vector is unpacked its registers take the same vector of the wavefront's next row: the loads
      // trickle out through the whole first sweep and have the rest of the row's work to arrive, while a row of
      // packed values and a row of fp32 values are all a lane ever holds.
      __builtin_amdgcn_sched_barrier(0);
      fetch1(c, znext);
      __builtin_amdgcn_sched_barrier(0);
    }
    float rs;
    if (ACT == ACT_RMS) {
      rs = 1.0f / __builtin_sqrtf(wave_sum(sum) * inv_n + eps);     // masked vectors hold zeros: they add nothing
    } else {
      const float mu = wave_sum(sum) * inv_n;
      float m2 = 0.0f;
#pragma unroll
      for (int c = 0; c < CH; c++)
#pragma unroll
        for (int v = 0; v < 8; v++) {
          const float d = a[c][v] - mu;
          a[c][v] = FULL ? d : (keep[c] ? d : 0.0f);
          m2 = __builtin_fmaf(a[c][v], a[c][v], m2);
        }
      rs = 1.0f / __builtin_sqrtf(wave_sum(m2) * inv_n + eps);
      if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
    }
    bf16_t* yr = Y + row * N;
#pragma unroll
    for (int c = 0; c < CH; c++) {
      const f32x4 g0 = gb[(c * 4 + 0) * 64 + lane], g1 = gb[(c * 4 + 1) * 64 + lane];
      bf16x8 o;
      if (ACT == ACT_RMS) {
#pragma unroll
        for (int v = 0; v < 4; v++) {
          o[v] = (bf16_t)(a[c][v] * rs * g0[v]);
          o[v + 4] = (bf16_t)(a[c][v + 4] * rs * g1[v]);
        }
      } else {
        const f32x4 b0 = gb[(c * 4 + 2) * 64 + lane], b1 = gb[(c * 4 + 3) * 64 + lane];
#pragma unroll
        for (int v = 0; v < 4; v++) {
          o[v] = (bf16_t)__builtin_fmaf(a[c][v] * rs, g0[v], b0[v]);
          o[v + 4] = (bf16_t)__builtin_fmaf(a[c][v + 4] * rs, g1[v], b1[v]);
        }
      }
      if (FULL) {
        bf16_t* yc = yr + c * 512;
        asm("" : "+s"(yc));
        __builtin_nontemporal_store(o, reinterpret_cast<bf16x8*>(yc + lane * 8));
      } else if (keep[c]) {
        *reinterpret_cast<bf16x8*>(yr + voff[c]) = o;
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the LDS reads of later vectors from being hoisted (registers)
    }
  }
}

// ------------------------------------------------------------------------------------------------
// sum of two values over a workgroup of NW wavefronts; `red` is this call's LDS slot ([NW][2] of C)
template <class C, int NW> __device__ __forceinline__ void wg_sum2(C& a, C& b, C (*red)[2]) {
  a = wave_sum(a);
  b = wave_sum(b);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[wave][0] = a; red[wave][1] = b; }
  __syncthreads();
  if constexpr (sizeof(C) == 4 && NW <= 16) {
    // lane w of every row of 16 lanes takes wavefront w's pair; one row sum finishes both totals
    const int l = threadIdx.x & 15;
    a = l < NW ? red[l < NW ? l : 0][0] : (C)0;
    b = l < NW ? red[l < NW ? l : 0][1] : (C)0;
    a = row16_sum(a);
    b = row16_sum(b);
  } else {
    a = red[0][0];
    b = red[0][1];
#pragma unroll
    for (int w = 1; w < NW; w++) { a += red[w][0]; b += red[w][1]; }
  }
}

// B1a (two-kernel path): c1_i = mean_j g_ij, c2_i = mean_j g_ij Ahat_ij with g = dY gamma.
template <class T, int V>
__global__ __launch_bounds__(256) void b1a_kernel(int64_t M, int64_t N, const T* __restrict__ dY,
                                                  const T* __restrict__ Z, const float* __restrict__ gamma,
                                                  const float* __restrict__ mean, const float* __restrict__ rstd,
                                                  typename ComputeOf<T>::type* __restrict__ c12) {
  typedef typename ComputeOf<T>::type C;
  __shared__ C red[2][4][2];
  int par = 0;
  for (int64_t row = blockIdx.x; row < M; row += gridDim.x, par ^= 1) {
    const C mu = (C)mean[row], rs = (C)rstd[row];
    C s1 = 0, s2 = 0;
    for (int64_t col = (int64_t)threadIdx.x * V; col < N; col += 256 * V) {
      C dy[V], z[V];
      VecIO<T, V>::load(dY + row * N + col, dy);
      VecIO<T, V>::load(Z + row * N + col, z);
#pragma unroll
      for (int v = 0; v < V; v++) {
        const C g = dy[v] * (C)gamma[col + v];
        const C ah = (gelu<C>(z[v]) - mu) * rs;
        s1 += g;
        s2 += g * ah;
      }
    }
    wg_sum2<C, 4>(s1, s2, red[par]);
    if (threadIdx.x == 0) { c12[row] = s1 / (C)N; c12[M + row] = s2 / (C)N; }
  }
}

// B1b (two-kernel path): dZ and column partials, given c1 and c2.
template <class T, int V>
__global__ __launch_bounds__(256) void b1b_kernel(int64_t M, int64_t N, int64_t ldz, int rows_per_group, int strips,
                                                  const T* __restrict__ dY, const T* __restrict__ Z,
                                                  const float* __restrict__ gamma, const float* __restrict__ mean,
                                                  const float* __restrict__ rstd,
                                                  const typename ComputeOf<T>::type* __restrict__ c12,
                                                  T* __restrict__ dZ, typename ComputeOf<T>::type* __restrict__ colpart) {
  typedef typename ComputeOf<T>::type C;
  const int strip = blockIdx.x % strips;
  const int64_t grp = blockIdx.x / strips;
  const int64_t col = ((int64_t)strip * 256 + threadIdx.x) * V;
  if (col >= N) return;
  C gm[V], accb[V], accg[V], accz[V];
#pragma unroll
  for (int v = 0; v < V; v++) { gm[v] = (C)gamma[col + v]; accb[v] = 0; accg[v] = 0; accz[v] = 0; }
  const int64_t r0 = grp * rows_per_group;
  int64_t r1 = r0 + rows_per_group;
  if (r1 > M) r1 = M;
#pragma unroll 2
  for (int64_t r = r0; r < r1; r++) {
    C dy[V], z[V], dz[V];
    VecIO<T, V>::load(dY + r * N + col, dy);
    VecIO<T, V>::load(Z + r * N + col, z);
    const C mu = (C)mean[r], rs = (C)rstd[r], c1 = c12[r], c2 = c12[M + r];
#pragma unroll
    for (int v = 0; v < V; v++) {
      C Phi, phi;
      Gauss<C>::eval(z[v], Phi, phi);
      const C ah = (Gauss<C>::gelu_of(z[v], Phi) - mu) * rs;
      const C g = dy[v] * gm[v];
      dz[v] = rs * (g - c1 - ah * c2) * (Phi + z[v] * phi);
      accb[v] += dy[v];
      accg[v] += dy[v] * ah;
      accz[v] += dz[v];
    }
    VecIO<T, V>::store(dZ + r * ldz + col, dz);
  }
#pragma unroll
  for (int v = 0; v < V; v++) {
    colpart[(grp * 3 + 0) * N + col + v] = accb[v];
    colpart[(grp * 3 + 1) * N + col + v] = accg[v];
    colpart[(grp * 3 + 2) * N + col + v] = accz[v];
  }
}

// ------------------------------------------------------------------------------------------------
// B1 fused: one pass, the row held in registers (S strips of NT*V columns, NT threads).  A workgroup walks rows
// blockIdx.x, blockIdx.x + gridDim.x, ... ; two rows of loads are in flight while a row is processed; one barrier
// per row (the LDS exchange slot alternates between consecutive rows).
template <class T, int V> struct RawVec;
template <> struct RawVec<float, 4> { typedef f32x4 type; };
template <> struct RawVec<float, 1> { typedef float type; };
template <> struct RawVec<bf16_t, 8> { typedef bf16x8 type; };
template <> struct RawVec<bf16_t, 1> { typedef bf16_t type; };

// Row data is used once per pass and is far larger than the caches: loads and stores of the big row-major
// tensors carry the non-temporal hint.
template <class T, int V> __device__ __forceinline__ typename RawVec<T, V>::type raw_load(const T* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const typename RawVec<T, V>::type*>(p));
}
template <class T, int V, class C> __device__ __forceinline__ C raw_get(const typename RawVec<T, V>::type& r, int v) {
  if constexpr (V == 1) return (C)to_f32<T>(r); else return (C)to_f32<T>(r[v]);
}
template <class T, int V> __device__ __forceinline__ typename RawVec<T, V>::type raw_zero() {
  typename RawVec<T, V>::type r;
  if constexpr (V == 1) r = (T)0.0f; else { for (int v = 0; v < V; v++) r[v] = (T)0.0f; }
  return r;
}

// TAB (bf16 only): Phi and z phi(z) come from the LDS table (exact for bf16 arguments) instead of the polynomial
// and the hardware exponential.  The backward pass must evaluate GELU exactly as the forward pass that produced
// mean and rstd did - for a constant row, rstd = eps^-1/2 multiplies any difference between the two into Ahat -
// so the launcher selects TAB if and only if the forward pass normalised with the table.
// BLK (16-byte vectors, one strip): dZ is written as [M / 32][N / 32] blocks of 32 x 32 elements, each block row-major
// (what the tuned dX and dW kernels read best, see gemm_bf16.hip).  A row's 16 bytes per lane are then 64-byte pieces,
// each half of a 128-byte line whose other half belongs to the next row: the group walks rows in neighbouring pairs,
// parks both rows' vectors in a per-wave LDS area and stores whole lines (lanes 8j .. 8j+3 the even row's piece j,
// lanes 8j+4 .. 8j+7 the odd row's).  Half-line stores straight from the registers cost the phase a third of its
// bandwidth (0.55 -> 0.73 ms on 65536 x 8192), halves merged in the L2 still a tenth.
template <class T, int V, int S, int NT, bool TAB, bool BLK = false>
__global__ __launch_bounds__(NT) void b1_fused_kernel(int64_t M, int64_t N, int64_t ldz, const T* __restrict__ dY,
                                                       const T* __restrict__ Z, const float* __restrict__ gamma,
                                                       const float* __restrict__ mean, const float* __restrict__ rstd,
                                                       T* __restrict__ dZ,
                                                       typename ComputeOf<T>::type* __restrict__ colpart) {
  typedef typename ComputeOf<T>::type C;
  typedef typename RawVec<T, V>::type raw_t;
  typedef GaussTable<true> GT;
  typedef __attribute__((address_space(3))) f32x2 lds_f32x2;
  static_assert(!BLK || (V * sizeof(T) == 16 && S == 1), "blocked output: 16-byte vectors, one strip");
  constexpr bool blocked = BLK;
  __shared__ C red[2][NT / 64][2];
  __shared__ __attribute__((aligned(8))) float gtab[TAB ? 2 * GT::kEntries : 2];
  __shared__ __attribute__((aligned(16))) raw_t park[BLK ? NT / 64 : 1][2][BLK ? 64 : 1];   // [wave][row of the pair][lane]
  uint32_t gorg = 0;
  if (TAB) {
    GT::build(gtab, threadIdx.x, NT);
    gorg = GT::origin((uint32_t)(uintptr_t)(const lds_f32x2*)gtab);
    __syncthreads();
  }
  int64_t col[S];
  bool ok[S];
  C gm[S][V], accb[S][V], accg[S][V], accz[S][V];
#pragma unroll
  for (int s = 0; s < S; s++) {
    col[s] = ((int64_t)s * NT + threadIdx.x) * V;
    ok[s] = col[s] < N;
#pragma unroll
    for (int v = 0; v < V; v++) {
      gm[s][v] = ok[s] ? (C)gamma[col[s] + v] : (C)0;
      accb[s][v] = 0; accg[s][v] = 0; accz[s][v] = 0;
    }
  }
  // Two rows are kept in flight: buffers 0 and 1 hold the raw rows r and r + G (G = gridDim.x; r and r + 1 where dZ
  // is blocked); as soon as a buffer has been unpacked its refill with the row 2G further on is issued, ahead of that
  // row's barrier and second phase.
  raw_t bdy[2][S], bz[2][S];
  const int64_t G = gridDim.x;
  auto fetch = [&](int buf, int64_t r) {
    if (r < M) {
#pragma unroll
      for (int s = 0; s < S; s++) {
        if (ok[s]) { bdy[buf][s] = raw_load<T, V>(dY + r * N + col[s]); bz[buf][s] = raw_load<T, V>(Z + r * N + col[s]); }
      }
    }
  };
#pragma unroll
  for (int buf = 0; buf < 2; buf++)
#pragma unroll
    for (int s = 0; s < S; s++) { bdy[buf][s] = raw_zero<T, V>(); bz[buf][s] = raw_zero<T, V>(); }
  // Row-major dZ: the group walks rows b, b + G, b + 2G, ... .  Blocked dZ: rows 2b, 2b + 1, then 2G further on - the
  // two rows in flight are neighbours, so the two 64-byte halves of every line of dZ leave the same compute unit
  // within one row time and merge in its L2 (M is even where dZ is blocked).
  const int64_t first = blocked ? 2 * (int64_t)blockIdx.x : (int64_t)blockIdx.x;
  const int64_t second = blocked ? 1 : G;
  fetch(0, first);
  fetch(1, first + second);

  const C inv_n = (C)1 / (C)N;
  auto process = [&](int buf, int64_t row) {
    const C mu = (C)mean[row], rs = (C)rstd[row];
    const C nmr = -mu * rs;
    C ah[S][V], gp[S][V], g[S][V];
    C s1 = 0, s2 = 0;
#pragma unroll
    for (int s = 0; s < S; s++)
#pragma unroll
      for (int v = 0; v < V; v++) {
        const C z = raw_get<T, V, C>(bz[buf][s], v);
        const C dy = raw_get<T, V, C>(bdy[buf][s], v);
        if constexpr (TAB) {
          const uint32_t zbits = __builtin_bit_cast(uint32_t, (float)z) >> 16;      // the bf16 bits of z
          const f32x2 e = *(const lds_f32x2*)(uintptr_t)GT::address_of(zbits, gorg);
          const float Phi = 0.5f + GT::with_sign_of(e[0], (float)z);
          ah[s][v] = ((float)z * Phi) * rs + nmr;
          gp[s][v] = (Phi + GT::with_sign_of(e[1], (float)z)) * rs;
        } else {
          C Phi, phi;
          Gauss<C>::eval(z, Phi, phi);
          ah[s][v] = Gauss<C>::gelu_of(z, Phi) * rs + nmr;   // (A - mean) rstd, one fused multiply-add
          gp[s][v] = (Phi + z * phi) * rs;
        }
        g[s][v] = dy * gm[s][v];
        s1 += g[s][v];
        s2 += g[s][v] * ah[s][v];
        accb[s][v] += dy;
        accg[s][v] += dy * ah[s][v];
      }
    fetch(buf, row + 2 * G);
    wg_sum2<C, NT / 64>(s1, s2, red[buf]);
    const C c1 = s1 * inv_n, c2 = s2 * inv_n;
#pragma unroll
    for (int s = 0; s < S; s++) {
      C dz[V];
#pragma unroll
      for (int v = 0; v < V; v++) {
        dz[v] = (g[s][v] - c1 - ah[s][v] * c2) * gp[s][v];
        accz[s][v] += dz[v];
      }
      typename RawVec<T, V>::type o;
      if constexpr (V == 1) o = to_storage<T, C>(dz[0]); else { for (int v = 0; v < V; v++) o[v] = to_storage<T, C>(dz[v]); }
      if constexpr (BLK) {
        // (every lane takes part in the stores, also one whose own columns lie past the end of the row: the pieces it
        //  stores belong to other lanes' columns)
        const int wv = threadIdx.x >> 6, ln = threadIdx.x & 63;
        if (ok[s]) park[wv][buf][ln] = o;
        if (buf == 1) {
          // this wave's 16 pieces per row (piece = 4 lanes = 32 columns = one block): two stores of 8 whole lines
          const int64_t even = row - 1;
#pragma unroll
          for (int half = 0; half < 2; half++) {
            const int j = half * 8 + (ln >> 3), i = ln & 7;
            const int64_t nb = (int64_t)wv * 16 + j;                       // block column of piece j
            if (nb * 32 < N) {                                             // N is a multiple of 32: a piece is whole or absent
              const raw_t v = park[wv][i >> 2][4 * j + (i & 3)];
              const int64_t at = (((even >> 5) * (N >> 5) + nb) << 10) + ((even & 31) << 5) + i * 8;
              __builtin_nontemporal_store(v, reinterpret_cast<raw_t*>(dZ + at));
            }
          }
        }
      } else if (ok[s]) {
        __builtin_nontemporal_store(o, reinterpret_cast<typename RawVec<T, V>::type*>(dZ + row * ldz + col[s]));
      }
    }
  };
  for (int64_t row = first; row < M; row += 2 * G) {
    process(0, row);
    if (row + second < M) process(1, row + second);
  }
#pragma unroll
  for (int s = 0; s < S; s++)
    if (ok[s]) {
#pragma unroll
      for (int v = 0; v < V; v++) {
        colpart[((int64_t)blockIdx.x * 3 + 0) * N + col[s] + v] = accb[s][v];
        colpart[((int64_t)blockIdx.x * 3 + 1) * N + col[s] + v] = accg[s][v];
        colpart[((int64_t)blockIdx.x * 3 + 2) * N + col[s] + v] = accz[s][v];
      }
    }
}

// ------------------------------------------------------------------------------------------------
// B2: colpart [groups][3][N] -> dbeta, dgamma, db.  64 consecutive columns per workgroup (coalesced), the groups
// dealt over the 16 wavefronts, four independent partial sums per thread so that several loads are in flight
// (the phase is pure latency: a few tens of MB), fp64 sums in a fixed order.
// (nwhich = gridDim.y kinds of partial per group, colpart [groups][nwhich][N]; kind w goes to out_w)
template <class C>
__device__ __forceinline__ void b2_columns(int64_t N, int groups, int nwhich, const C* __restrict__ colpart, int cblock,
                                           int which, float* __restrict__ out, double (*red)[64]) {
  constexpr int kSlices = 16;
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int64_t col = (int64_t)cblock * 64 + lane;
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
  if (col < N) {
    const C* src = colpart + (int64_t)which * N + col;
    const int64_t gstride = (int64_t)nwhich * N;
    int g = slice;
    for (; g + 3 * kSlices < groups; g += 4 * kSlices) {
      const C v0 = src[(int64_t)g * gstride], v1 = src[(int64_t)(g + kSlices) * gstride];
      const C v2 = src[(int64_t)(g + 2 * kSlices) * gstride], v3 = src[(int64_t)(g + 3 * kSlices) * gstride];
      a0 += (double)v0; a1 += (double)v1; a2 += (double)v2; a3 += (double)v3;
    }
    for (; g < groups; g += kSlices) a0 += (double)src[(int64_t)g * gstride];
  }
  red[slice][lane] = (a0 + a1) + (a2 + a3);
  __syncthreads();
  if (slice == 0 && col < N) {
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < kSlices; w++) t += red[w][lane];
    out[col] = (float)t;
  }
}

template <class C>
__global__ __launch_bounds__(1024) void b2_kernel(int64_t N, int groups, const C* __restrict__ colpart,
                                                  float* __restrict__ dbeta, float* __restrict__ dgamma,
                                                  float* __restrict__ db) {
  __shared__ double red[16][64];
  const int which = blockIdx.y;
  b2_columns<C>(N, groups, (int)gridDim.y, colpart, (int)blockIdx.x, which,
                which == 0 ? dbeta : (which == 1 ? dgamma : db), red);
}

// The tail of a bf16 backward pass in one launch, for shapes where the contractions leave split reductions behind:
// workgroups [0, a.blocks) and [a.blocks, a.blocks + b.blocks) add the fp32 partial products of up to two outputs
// (4096 elements per workgroup, partials summed in index order, one rounding to bf16), the remaining 3 ceil(N / 64)
// workgroups finish the column sums exactly as b2_kernel does.  Small dependent launches cost a few microseconds each
// whatever they do, which is what this saves for mid-sized layers.
__global__ __launch_bounds__(1024) void finish_kernel(TailSums j) {
  __shared__ double red[16][64];
  int id = (int)blockIdx.x;
  for (int k = 0; k < 2; k++) {
    if (id < j.blocks[k]) {
      const int64_t i = ((int64_t)id * 1024 + threadIdx.x) * 4;
      if (i >= j.n[k]) return;
      const float* part = j.part[k];
      f32x4 acc = *reinterpret_cast<const f32x4*>(part + i);
      for (int q = 1; q < j.parts[k]; q++) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(part + (int64_t)q * j.n[k] + i);
        acc[0] += t[0]; acc[1] += t[1]; acc[2] += t[2]; acc[3] += t[3];
      }
      bf16x4 o;
      o[0] = (bf16_t)acc[0]; o[1] = (bf16_t)acc[1]; o[2] = (bf16_t)acc[2]; o[3] = (bf16_t)acc[3];
      *reinterpret_cast<bf16x4*>(static_cast<bf16_t*>(j.out[k]) + i) = o;
      return;
    }
    id -= j.blocks[k];
  }
  const int cblocks = (int)((j.N + 63) / 64);
  const int which = id / cblocks;
  b2_columns<float>(j.N, j.groups, 3, j.colpart, id % cblocks, which,
                    which == 0 ? j.dbeta : (which == 1 ? j.dgamma : j.db), red);
}


// ------------------------------------------------------------------------------------------------
// Stand-alone row normalisation for any shape and both storage types: one workgroup per row at a time, the row read
// from memory (and then from the caches) once per pass - sum, squared deviations, output - as in the paper's
// two-step LayerNorm and strided RMSNorm kernels.  MODE: ACT_NONE LayerNorm (writes mean, rstd), ACT_RMS RMSNorm.
template <class T, int V, int MODE>
__global__ __launch_bounds__(256) void norm_wg_kernel(int64_t M, int64_t N, float eps, const T* __restrict__ A,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      T* __restrict__ Y, float* __restrict__ mean, float* __restrict__ rstd) {
  typedef typename ComputeOf<T>::type C;
  __shared__ C red[2][4][2];
  for (int64_t row = blockIdx.x; row < M; row += gridDim.x) {
    const T* a = A + row * N;
    C s1 = 0, s2 = 0;
    for (int64_t col = (int64_t)threadIdx.x * V; col < N; col += 256 * V) {
      C x[V];
      VecIO<T, V>::load(a + col, x);
#pragma unroll
      for (int v = 0; v < V; v++) { s1 += x[v]; s2 += x[v] * x[v]; }
    }
    wg_sum2<C, 4>(s1, s2, red[0]);
    C mu = 0, rs;
    if (MODE == ACT_RMS) {
      rs = (C)1 / sqrt(s2 / (C)N + (C)eps);
    } else {
      mu = s1 / (C)N;
      C d2 = 0, dummy = 0;
      for (int64_t col = (int64_t)threadIdx.x * V; col < N; col += 256 * V) {
        C x[V];
        VecIO<T, V>::load(a + col, x);
#pragma unroll
        for (int v = 0; v < V; v++) { const C d = x[v] - mu; d2 += d * d; }
      }
      wg_sum2<C, 4>(d2, dummy, red[1]);
      rs = (C)1 / sqrt(d2 / (C)N + (C)eps);
      if (threadIdx.x == 0) { mean[row] = (float)mu; rstd[row] = (float)rs; }
    }
    for (int64_t col = (int64_t)threadIdx.x * V; col < N; col += 256 * V) {
      C x[V], y[V];
      VecIO<T, V>::load(a + col, x);
#pragma unroll
      for (int v = 0; v < V; v++) {
        if (MODE == ACT_RMS) y[v] = x[v] * rs * (C)gamma[col + v];
        else y[v] = (x[v] - mu) * rs * (C)gamma[col + v] + (C)beta[col + v];
      }
      VecIO<T, V>::store(Y + row * N + col, y);
    }
    __syncthreads();   // the exchange slots are reused by the next row
  }
}

// Column sums of a row-major matrix, first stage: workgroup g sums rows g, g + G, ... of a strip of 256 V columns
// into colpart[g][N] (arithmetic type); b2_kernel finishes them.  Coalesced along the row, no atomics.
// BLK: the matrix is stored in 32 x 32 blocks (see gemm_bf16.hip); a lane's 16 bytes are then a quarter of a 64-byte
// piece, and the group walks rows in neighbouring pairs, whose pieces share a line (M even).
template <class T, int V, bool BLK = false>
__global__ __launch_bounds__(256) void colsum_partial_kernel(int64_t M, int64_t N, int strips, int groups,
                                                             const T* __restrict__ G,
                                                             typename ComputeOf<T>::type* __restrict__ colpart) {
  typedef typename ComputeOf<T>::type C;
  const int strip = blockIdx.x % strips;
  const int grp = blockIdx.x / strips;
  const int64_t col = ((int64_t)strip * 256 + threadIdx.x) * V;
  if (col >= N) return;
  C acc[V];
#pragma unroll
  for (int v = 0; v < V; v++) acc[v] = 0;
  if constexpr (BLK) {
    const int64_t cb = ((col >> 5) << 10) + (col & 31);
#pragma unroll 2
    for (int64_t r = 2 * (int64_t)grp; r < M; r += 2 * (int64_t)groups) {
      const T* base = G + (((r >> 5) * (N >> 5)) << 10) + ((r & 31) << 5) + cb;
      C x[V], y[V];
      VecIO<T, V>::load(base, x);
      VecIO<T, V>::load(base + 32, y);     // row r + 1 (r is even: same block row)
#pragma unroll
      for (int v = 0; v < V; v++) acc[v] += x[v] + y[v];
    }
  } else {
#pragma unroll 4
    for (int64_t r = grp; r < M; r += groups) {
      C x[V];
      VecIO<T, V>::load(G + r * N + col, x);
#pragma unroll
      for (int v = 0; v < V; v++) acc[v] += x[v];
    }
  }
#pragma unroll
  for (int v = 0; v < V; v++) colpart[(int64_t)grp * N + col + v] = acc[v];
}

// H = SiLU(G) * U, element by element (the gated feed-forward block's activation); H may be G or U.
template <class T, int V>
__global__ __launch_bounds__(256) void silu_mul_kernel(int64_t n, const T* G, const T* U, T* H) {
  typedef typename ComputeOf<T>::type C;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * V; i < n; i += (int64_t)gridDim.x * 256 * V) {
    C g[V], u[V], h[V];
    VecIO<T, V>::load(G + i, g);
    VecIO<T, V>::load(U + i, u);
#pragma unroll
    for (int v = 0; v < V; v++) {
      if constexpr (sizeof(C) == 8) h[v] = g[v] / (1.0 + exp(-g[v])) * u[v];
      else h[v] = g[v] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896340736f * g[v])) * u[v];
    }
    VecIO<T, V>::store(H + i, h);
  }
}

// vector width usable for rows of length N starting at `base` (every row start must be aligned)
template <class T> int vec_width(const void* a, const void* b, const void* c, int64_t N) {
  constexpr int V = 16 / (int)sizeof(T);
  const uintptr_t m = (uintptr_t)a | (uintptr_t)b | (uintptr_t)c;
  return (N % V == 0 && m % 16 == 0) ? V : 1;
}

template <class T> void f2_impl(int64_t M, int64_t N, const void* Z, const float* mean, const float* rstd,
                                const float* gamma, const float* beta, void* Y, hipStream_t s) {
  constexpr int VMAX = 16 / (int)sizeof(T);
  const int V = vec_width<T>(Z, Y, nullptr, N);
  const int strips = (int)((N + 256 * (int64_t)V - 1) / (256 * (int64_t)V));
  // 16 rows per workgroup keep gamma and beta in registers across rows; fewer where the matrix is so small that the
  // chip would otherwise see only a handful of workgroups
  int64_t rows_per_wg = M * strips / 2048;
  rows_per_wg = rows_per_wg < 1 ? 1 : (rows_per_wg > 16 ? 16 : rows_per_wg);
  const int64_t blocks = (int64_t)strips * ((M + rows_per_wg - 1) / rows_per_wg);
  if (V == VMAX)
    hipLaunchKernelGGL((f2_kernel<T, VMAX>), dim3((unsigned)blocks), dim3(256), 0, s, M, N, (int)rows_per_wg, strips,
                       (const T*)Z, mean, rstd, gamma, beta, (T*)Y);
  else
    hipLaunchKernelGGL((f2_kernel<T, 1>), dim3((unsigned)blocks), dim3(256), 0, s, M, N, (int)rows_per_wg, strips,
                       (const T*)Z, mean, rstd, gamma, beta, (T*)Y);
}

template <class T> void b1a_impl(int64_t M, int64_t N, const void* dY, const void* Z, const float* gamma,
                                 const float* mean, const float* rstd, void* c12, hipStream_t s) {
  typedef typename ComputeOf<T>::type C;
  constexpr int VMAX = 16 / (int)sizeof(T);
  const int V = vec_width<T>(dY, Z, nullptr, N);
  const unsigned blocks = (unsigned)(M < 4096 ? M : 4096);
  if (V == VMAX)
    hipLaunchKernelGGL((b1a_kernel<T, VMAX>), dim3(blocks), dim3(256), 0, s, M, N, (const T*)dY, (const T*)Z, gamma,
                       mean, rstd, (C*)c12);
  else
    hipLaunchKernelGGL((b1a_kernel<T, 1>), dim3(blocks), dim3(256), 0, s, M, N, (const T*)dY, (const T*)Z, gamma, mean,
                       rstd, (C*)c12);
}

template <class T> void b1b_impl(int64_t M, int64_t N, int64_t ldz, int rows_per_group, int groups, const void* dY, const void* Z,
                                 const float* gamma, const float* mean, const float* rstd, const void* c12, void* dZ,
                                 void* colpart, hipStream_t s) {
  typedef typename ComputeOf<T>::type C;
  constexpr int VMAX = 16 / (int)sizeof(T);
  const int V = (ldz % VMAX == 0) ? vec_width<T>(dY, Z, dZ, N) : 1;
  const int strips = (int)((N + 256 * (int64_t)V - 1) / (256 * (int64_t)V));
  const int64_t blocks = (int64_t)strips * groups;
  if (V == VMAX)
    hipLaunchKernelGGL((b1b_kernel<T, VMAX>), dim3((unsigned)blocks), dim3(256), 0, s, M, N, ldz, rows_per_group, strips,
                       (const T*)dY, (const T*)Z, gamma, mean, rstd, (const C*)c12, (T*)dZ, (C*)colpart);
  else
    hipLaunchKernelGGL((b1b_kernel<T, 1>), dim3((unsigned)blocks), dim3(256), 0, s, M, N, ldz, rows_per_group, strips,
                       (const T*)dY, (const T*)Z, gamma, mean, rstd, (const C*)c12, (T*)dZ, (C*)colpart);
}

// Launch shapes of the fused kernel (threads NT, strips S): full-width vectors use one strip and 256, 512
// or 1024 threads; the scalar (unaligned rows) variant also has a two-strip, 1024-thread shape.
struct FusedShape { int nt, s; };
inline bool fused_shape(int64_t N, int V, bool vec, FusedShape* out) {
  const int64_t per_thread = (N + V - 1) / V;   // vectors per row
  const int nts[3] = {256, 512, 1024};
  for (int i = 0; i < 3; i++)
    if (per_thread <= nts[i]) { out->nt = nts[i]; out->s = 1; return true; }
  if (!vec && per_thread <= 2048) { out->nt = 1024; out->s = 2; return true; }
  return false;
}

template <class T, bool TAB> void b1_fused_impl(int64_t M, int64_t N, int64_t ldz, int groups, bool blocked, const void* dY, const void* Z,
                                                const float* gamma, const float* mean, const float* rstd, void* dZ,
                                                void* colpart, hipStream_t s) {
  typedef typename ComputeOf<T>::type C;
  constexpr int VMAX = 16 / (int)sizeof(T);
  const int V = vec_width<T>(dY, Z, dZ, N);
  FusedShape fs;
  if (!fused_shape(N, V, V == VMAX, &fs)) return;   // callers check b1_fused_supported first
#define FDL_B1F(VV, SS, NTT)                                                                                       \
  hipLaunchKernelGGL((b1_fused_kernel<T, VV, SS, NTT, TAB>), dim3((unsigned)groups), dim3(NTT), 0, s, M, N, ldz,      \
                     (const T*)dY, (const T*)Z, gamma, mean, rstd, (T*)dZ, (C*)colpart)
#define FDL_B1F_BLK(NTT)                                                                                           \
  hipLaunchKernelGGL((b1_fused_kernel<T, VMAX, 1, NTT, TAB, true>), dim3((unsigned)groups), dim3(NTT), 0, s, M, N,  \
                     ldz, (const T*)dY, (const T*)Z, gamma, mean, rstd, (T*)dZ, (C*)colpart)
  if (V == VMAX && blocked) {
    if constexpr (sizeof(T) == 2) {
      if (fs.nt == 256) FDL_B1F_BLK(256); else if (fs.nt == 512) FDL_B1F_BLK(512); else FDL_B1F_BLK(1024);
    }
  } else if (V == VMAX) {
    if (fs.nt == 256) FDL_B1F(VMAX, 1, 256); else if (fs.nt == 512) FDL_B1F(VMAX, 1, 512); else FDL_B1F(VMAX, 1, 1024);
  } else {
    if (fs.s == 2) FDL_B1F(1, 2, 1024);
    else if (fs.nt == 256) FDL_B1F(1, 1, 256); else if (fs.nt == 512) FDL_B1F(1, 1, 512); else FDL_B1F(1, 1, 1024);
  }
#undef FDL_B1F_BLK
#undef FDL_B1F
}

}  // namespace

void launch_stats_finalize(const void* part, int tiles, int tile_w, int64_t M, int64_t N, float eps, float* mean,
                           float* rstd, hipStream_t s) {
  const unsigned blocks = (unsigned)((M + 15) / 16);   // sixteen lanes per row
  hipLaunchKernelGGL(stats_finalize_kernel, dim3(blocks), dim3(256), 0, s, (const f32x2*)part, tiles, tile_w, M, N, eps,
                     mean, rstd);
}

void launch_f2(int dt, int64_t M, int64_t N, const void* Zsave, const float* mean, const float* rstd,
               const float* gamma, const float* beta, void* Y, hipStream_t s) {
  if (dt == kF32) f2_impl<float>(M, N, Zsave, mean, rstd, gamma, beta, Y, s);
  else f2_impl<bf16_t>(M, N, Zsave, mean, rstd, gamma, beta, Y, s);
}

// one instantiation: gamma/beta (4 KB per 512 columns) plus the Phi table can exceed the default 64 KB of dynamic LDS
template <int CH, bool FULL, int NT, int ACT>
void launch_f2_rows_one(int64_t wgs, hipStream_t s, int64_t M, int64_t N, float eps, const bf16_t* Z, const float* gamma,
                        const float* beta, bf16_t* Y, float* mean, float* rstd) {
  constexpr size_t kLds = (size_t)CH * 4096 + GaussTable<false>::kBytes;
  static OnceFlags configured;
  auto kern = f2_rows_kernel<CH, FULL, NT, ACT>;
  if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)kLds, &configured)) return;
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(NT), kLds, s, M, N, eps, Z, gamma, beta, Y, mean, rstd);
}

bool f2_rows_supported(int dt, int64_t N) { return dt == kBF16 && N % 8 == 0 && N <= 8192; }

template <int ACT>
void launch_rows_act(int64_t M, int64_t N, float eps, const void* Zsave, const float* gamma, const float* beta, void* Y,
                     float* mean, float* rstd, hipStream_t s) {
  int ch = 2;
  while (ch * 512 < N) ch *= 2;
  const bool full = N == (int64_t)ch * 512;
  const int nt = (!full && ch == 16) ? 256 : 512;
  // a workgroup of the widest variant fills a CU's register file; narrower rows leave room for more of them
  const int64_t per_wg = nt / 64;
  int64_t wgs = (M + per_wg - 1) / per_wg;
  DeviceInfo di;
  if (!device_info(&di)) return;
  const int64_t cap = (int64_t)di.cus * (16 / ch);
  if (wgs > cap) wgs = cap;
#define FDL_F2R(CHH, FULL, NTT)                                                                                    \
  launch_f2_rows_one<CHH, FULL, NTT, ACT>(wgs, s, M, N,                                                                 \
                     eps, (const bf16_t*)Zsave, gamma, beta, (bf16_t*)Y, mean, rstd)
  if (full) {
    if (ch == 2) FDL_F2R(2, true, 512); else if (ch == 4) FDL_F2R(4, true, 512);
    else if (ch == 8) FDL_F2R(8, true, 512); else FDL_F2R(16, true, 512);
  } else {
    if (ch == 2) FDL_F2R(2, false, 512); else if (ch == 4) FDL_F2R(4, false, 512);
    else if (ch == 8) FDL_F2R(8, false, 512); else FDL_F2R(16, false, 256);
  }
#undef FDL_F2R
}

void launch_f2_rows(int64_t M, int64_t N, float eps, const void* Zsave, const float* gamma, const float* beta, void* Y,
                    float* mean, float* rstd, hipStream_t s) {
  launch_rows_act<ACT_GELU>(M, N, eps, Zsave, gamma, beta, Y, mean, rstd, s);
}


bool rows_act_supported(int dt, int64_t N) { return f2_rows_supported(dt, N); }

template <class T, int MODE>
static void norm_wg_impl(int64_t M, int64_t N, float eps, const void* A, const float* gamma, const float* beta, void* Y,
                         float* mean, float* rstd, hipStream_t s) {
  constexpr int VMAX = 16 / (int)sizeof(T);
  const bool vec = N % VMAX == 0 && ((uintptr_t)A | (uintptr_t)Y) % 16 == 0;
  const unsigned blocks = (unsigned)(M < 8192 ? M : 8192);
  if (vec) hipLaunchKernelGGL((norm_wg_kernel<T, VMAX, MODE>), dim3(blocks), dim3(256), 0, s, M, N, eps, (const T*)A, gamma, beta, (T*)Y, mean, rstd);
  else hipLaunchKernelGGL((norm_wg_kernel<T, 1, MODE>), dim3(blocks), dim3(256), 0, s, M, N, eps, (const T*)A, gamma, beta, (T*)Y, mean, rstd);
}

// Y = LayerNorm(A) gamma + beta over the last dimension; mean, rstd [M] out
void launch_layernorm(int dt, int64_t M, int64_t N, float eps, const void* A, const float* gamma, const float* beta,
                      void* Y, float* mean, float* rstd, hipStream_t s) {
  if (rows_act_supported(dt, N)) launch_rows_act<ACT_NONE>(M, N, eps, A, gamma, beta, Y, mean, rstd, s);
  else if (dt == kF32) norm_wg_impl<float, ACT_NONE>(M, N, eps, A, gamma, beta, Y, mean, rstd, s);
  else norm_wg_impl<bf16_t, ACT_NONE>(M, N, eps, A, gamma, beta, Y, mean, rstd, s);
}

// Y = A (mean(A^2) + eps)^-1/2 weight over the last dimension
void launch_rmsnorm(int dt, int64_t M, int64_t N, float eps, const void* A, const float* weight, void* Y, hipStream_t s) {
  if (rows_act_supported(dt, N)) launch_rows_act<ACT_RMS>(M, N, eps, A, weight, weight, Y, nullptr, nullptr, s);
  else if (dt == kF32) norm_wg_impl<float, ACT_RMS>(M, N, eps, A, weight, weight, Y, nullptr, nullptr, s);
  else norm_wg_impl<bf16_t, ACT_RMS>(M, N, eps, A, weight, weight, Y, nullptr, nullptr, s);
}

// groups of the first stage of a column sum over M rows
int colsum_groups(int64_t M) { return (int)(M < 256 ? (M > 0 ? M : 1) : 256); }

// out[j] = sum_i G[i][j]; colpart: colsum_groups(M) * N values of the arithmetic type
void launch_colsum(int dt, int64_t M, int64_t N, const void* G, bool blocked, void* colpart, float* out, hipStream_t s) {
  const int groups = colsum_groups(M);
  const int vmax = dt == kF32 ? 4 : 8;
  const bool vec = N % vmax == 0 && (uintptr_t)G % 16 == 0;
  const int V = vec ? vmax : 1;
  const int strips = (int)((N + 256 * (int64_t)V - 1) / (256 * (int64_t)V));
  const dim3 grid((unsigned)(strips * groups));
  if (dt == kF32) {
    if (vec) hipLaunchKernelGGL((colsum_partial_kernel<float, 4>), grid, dim3(256), 0, s, M, N, strips, groups, (const float*)G, (double*)colpart);
    else hipLaunchKernelGGL((colsum_partial_kernel<float, 1>), grid, dim3(256), 0, s, M, N, strips, groups, (const float*)G, (double*)colpart);
    hipLaunchKernelGGL((b2_kernel<double>), dim3((unsigned)((N + 63) / 64), 1), dim3(1024), 0, s, N, groups, (const double*)colpart, out, out, out);
  } else {
    if (vec && blocked) hipLaunchKernelGGL((colsum_partial_kernel<bf16_t, 8, true>), grid, dim3(256), 0, s, M, N, strips, groups, (const bf16_t*)G, (float*)colpart);
    else if (vec) hipLaunchKernelGGL((colsum_partial_kernel<bf16_t, 8>), grid, dim3(256), 0, s, M, N, strips, groups, (const bf16_t*)G, (float*)colpart);
    else hipLaunchKernelGGL((colsum_partial_kernel<bf16_t, 1>), grid, dim3(256), 0, s, M, N, strips, groups, (const bf16_t*)G, (float*)colpart);
    hipLaunchKernelGGL((b2_kernel<float>), dim3((unsigned)((N + 63) / 64), 1), dim3(1024), 0, s, N, groups, (const float*)colpart, out, out, out);
  }
}

// H = SiLU(G) * U over n elements (H may alias G or U)
void launch_silu_mul(int dt, int64_t n, const void* G, const void* U, void* H, hipStream_t s) {
  const int vmax = dt == kF32 ? 4 : 8;
  const bool vec = n % vmax == 0 && ((uintptr_t)G | (uintptr_t)U | (uintptr_t)H) % 16 == 0;
  const int64_t per = 256 * (int64_t)(vec ? vmax : 1);
  int64_t blocks = (n + per - 1) / per;
  if (blocks > 16384) blocks = 16384;
  if (blocks < 1) blocks = 1;
  if (dt == kF32) {
    if (vec) hipLaunchKernelGGL((silu_mul_kernel<float, 4>), dim3((unsigned)blocks), dim3(256), 0, s, n, (const float*)G, (const float*)U, (float*)H);
    else hipLaunchKernelGGL((silu_mul_kernel<float, 1>), dim3((unsigned)blocks), dim3(256), 0, s, n, (const float*)G, (const float*)U, (float*)H);
  } else {
    if (vec) hipLaunchKernelGGL((silu_mul_kernel<bf16_t, 8>), dim3((unsigned)blocks), dim3(256), 0, s, n, (const bf16_t*)G, (const bf16_t*)U, (bf16_t*)H);
    else hipLaunchKernelGGL((silu_mul_kernel<bf16_t, 1>), dim3((unsigned)blocks), dim3(256), 0, s, n, (const bf16_t*)G, (const bf16_t*)U, (bf16_t*)H);
  }
}

void launch_b1a(int dt, int64_t M, int64_t N, const void* dY, const void* Zsave, const float* gamma, const float* mean,
                const float* rstd, void* c12, hipStream_t s) {
  if (dt == kF32) b1a_impl<float>(M, N, dY, Zsave, gamma, mean, rstd, c12, s);
  else b1a_impl<bf16_t>(M, N, dY, Zsave, gamma, mean, rstd, c12, s);
}

void launch_b1b(int dt, int64_t M, int64_t N, int64_t ldz, int rows_per_group, int groups, const void* dY, const void* Zsave,
                const float* gamma, const float* mean, const float* rstd, const void* c12, void* dZ, void* colpart,
                hipStream_t s) {
  if (dt == kF32) b1b_impl<float>(M, N, ldz, rows_per_group, groups, dY, Zsave, gamma, mean, rstd, c12, dZ, colpart, s);
  else b1b_impl<bf16_t>(M, N, ldz, rows_per_group, groups, dY, Zsave, gamma, mean, rstd, c12, dZ, colpart, s);
}

// dZ [M][ldz]: zero the surplus columns [N, ldz) of every row (padded mode of the fast contractions)
namespace {
__global__ __launch_bounds__(256) void zero_cols_kernel(unsigned short* __restrict__ dZ, int64_t M, int64_t N, int64_t ldz) {
  const int64_t w = ldz - N, n = M * w;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / w, c = i - r * w;
    dZ[r * ldz + N + c] = 0;
  }
}
}  // namespace
void launch_zero_cols_bf16(void* dZ, int64_t M, int64_t N, int64_t ldz, hipStream_t s) {
  if (ldz <= N || M <= 0) return;
  int64_t blocks = (M * (ldz - N) + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(zero_cols_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (unsigned short*)dZ, M, N, ldz);
}

// Whether rows can be read with full-width vectors depends on N only here (base pointers are required to be
// 16-byte aligned by the entry points).
bool b1_fused_supported(int dt, int64_t N) {
  const int vmax = dt == kF32 ? 4 : 8;
  const int V = (N % vmax == 0) ? vmax : 1;
  FusedShape fs;
  return fused_shape(N, V, V == vmax, &fs);
}

// Row groups (= workgroups) of the fused kernel.  Each group leaves 3 N partial column sums behind, so fewer groups
// mean less traffic for the phase and for the column reduction after it, while the rows in flight (two per group)
// must keep the memory system busy.  Measured: 256 groups are best once a row takes at least 512 lanes (with 1024
// threads a workgroup fills a CU's register file, all groups are resident at once and the rows in flight form one
// contiguous window); narrower rows need 512 groups, unless the matrix is so short that a group would walk fewer
// than 8 rows.
int b1_fused_groups(int dt, int64_t M, int64_t N) {
  const int vmax = dt == kF32 ? 4 : 8;
  const int V = (N % vmax == 0) ? vmax : 1;
  FusedShape fs;
  if (!fused_shape(N, V, V == vmax, &fs)) return 512;
  const int64_t lanes = (N + V - 1) / V;
  int64_t groups = lanes >= 512 ? 256 : 512;
  if (M / 8 < groups) groups = M / 8 < 256 ? 256 : M / 8;
  return (int)groups;
}

void launch_b1_fused(int dt, int64_t M, int64_t N, int64_t ldz, int groups, bool table, bool blocked, const void* dY,
                     const void* Zsave, const float* gamma, const float* mean, const float* rstd, void* dZ, void* colpart,
                     hipStream_t s) {
  const bool blk = blocked && dt == kBF16;
  if (dt == kF32) b1_fused_impl<float, false>(M, N, ldz, groups, false, dY, Zsave, gamma, mean, rstd, dZ, colpart, s);
  else if (table) b1_fused_impl<bf16_t, true>(M, N, ldz, groups, blk, dY, Zsave, gamma, mean, rstd, dZ, colpart, s);
  else b1_fused_impl<bf16_t, false>(M, N, ldz, groups, blk, dY, Zsave, gamma, mean, rstd, dZ, colpart, s);
}

void launch_b2(int dt, int64_t N, int groups, const void* colpart, float* dbeta, float* dgamma, float* db,
               hipStream_t s) {
  const dim3 grid((unsigned)((N + 63) / 64), 3);
  if (dt == kF32) hipLaunchKernelGGL((b2_kernel<double>), grid, dim3(1024), 0, s, N, groups, (const double*)colpart, dbeta, dgamma, db);
  else hipLaunchKernelGGL((b2_kernel<float>), grid, dim3(1024), 0, s, N, groups, (const float*)colpart, dbeta, dgamma, db);
}

// n[k] must be multiples of 4 (they are products of tile-aligned or 8-aligned dimensions on the bf16 tuned path).
void launch_finish(TailSums j, hipStream_t s) {
  unsigned blocks = 0;
  for (int k = 0; k < 2; k++) {
    j.blocks[k] = j.parts[k] > 0 ? (int)((j.n[k] / 4 + 1023) / 1024) : 0;
    blocks += (unsigned)j.blocks[k];
  }
  blocks += 3u * (unsigned)((j.N + 63) / 64);
  hipLaunchKernelGGL(finish_kernel, dim3(blocks), dim3(1024), 0, s, j);
}

}  // namespace fdl
