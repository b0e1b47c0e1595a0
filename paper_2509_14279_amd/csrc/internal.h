// Host-side declarations shared by the translation units of libfdl: the launch plan (which
// kernels run, how the workspace is carved up) and one launcher per phase of the block.
//
// Phases:  F1  Z = X W^T + b, Zsave, per-(row, column tile) partial statistics of GELU(Zsave)
//          FS  merge partial statistics -> mean, rstd
//          F2  Y = (GELU(Zsave) - mean) rstd gamma + beta
//              (bf16 fast path with rows that fit a wavefront's registers: F1 stores Zsave only, F2 takes the
//               statistics itself and FS is empty)
//          B1  dZ and the column partials of dbeta, dgamma, db  (B1a: row sums c1, c2 first)
//          B2  column partials -> dbeta, dgamma, db
//          B3  dX = dZ W            B4  dW = dZ^T X
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace fdl {

enum DType { kF32 = 0, kBF16 = 1 };

struct Plan {
  int dt;
  int64_t M, K, N;
  // forward
  int f1_fast;            // 1: bf16 fast MFMA kernel, 0: generic kernel
  int f2_rows;            // 1: F1 stores Zsave only; one kernel takes the row statistics and normalises (no FS)
  int f1_wb;              // generic kernel: 16x16 blocks per wave tile side (wave tile = 16*wb)
  int stat_tile_w;        // width of one partial-statistics column tile
  int stat_tiles;         // number of such tiles per row
  size_t off_part;        // float2 [stat_tiles][M]
  int f1_wt;              // 1: the fast kernel reads the weights from a transposed copy (large batches)
  size_t off_wt;          // bf16 [K][N], the last region of the forward workspace
  size_t fwd_bytes;       // (without the transposed weights: fwd_bytes - align256(N K 2), see fwd_bytes_plain)
  size_t fwd_bytes_plain; // forward workspace of the same plan with f1_wt = 0
  // backward
  int b1_fused;           // 1: one pass with the row held in registers; 0: B1a + B1b
  int b1_groups;          // number of row groups that produce column partials
  int b1_rows_per_group;  // B1b only
  int b3_fast, b4_fast;
  int b3_wb, b4_wb;
  int b4_split;           // split of the reduction over M in B4 (fast kernel)
  int64_t b4_fast_rows;   // rows of the reduction the fast kernel covers (the rest goes through the generic kernel)
  int pair;               // 1: dX and dW share one launch, their reductions split into pair_sa and pair_sb parts
  int pair_sa, pair_sb;
  int dz_blocked;         // 1: dZ lives in 32 x 32 blocks (fused row kernel -> tuned dX and dW kernels only)
  size_t off_dxpart;      // float [pair_sa][M][K] (pair_sa > 1)
  int pad;                // 1: padded mode of the fast contractions (N, K multiples of 8, not both of 256)
  int64_t ldz;            // pitch of the dZ buffer in elements (N, or N rounded up to 256 in padded mode)
  size_t off_wpad_f, off_bpad_f;   // forward: zero-padded copies of W [Np][Kp] and b [Np]
  size_t off_wpad_b;               // backward: zero-padded copy of W
  size_t off_xtail;       // forward: padded copy of X's last rows (ragged M on the fast path)
  size_t off_dz;          // T [M][N]
  size_t off_c12;         // C [2][M]
  size_t off_colpart;     // C [groups][3][N]
  size_t off_dwpart;      // float [split][N][K]
  size_t bwd_bytes;
  size_t bytes;           // max(fwd, bwd)
};

// Returns false when the shape or dtype is not supported.
bool make_plan(int dt, int64_t M, int64_t K, int64_t N, Plan* p);

// ---- per-device facts and per-call failure notes --------------------------------------------------
// Compute units and accelerator dies (each die has its own L2) of the calling thread's current device, queried from
// the runtime once per device.  Returns false (and leaves a note, see below) if the query fails.
struct DeviceInfo { int cus; int xcds; };
bool device_info(DeviceInfo* out);

// A launcher that cannot launch (a failed attribute call, a failed device query) prints the reason to stderr and
// leaves a note for the calling thread; the entry point turns a note into FDL_ERR_LAUNCH.
void note_failure(const char* what, hipError_t e);

// Raise the dynamic-LDS limit of a kernel once per device (flags: one byte per device ordinal, zero-initialised,
// owned by the caller - one array per kernel instantiation).  Safe to call from several host threads.
constexpr int kMaxDevices = 64;
struct OnceFlags { std::atomic<unsigned char> done[kMaxDevices]; };
bool ensure_dynamic_lds(const void* kernel, int bytes, OnceFlags* flags);

// ---- generic MFMA GEMM: C[i][j] = sum_r A(i,r) B(j,r), any shape, any alignment -----------------
// a_rc / b_rc: the operand is contiguous along the reduction index r (element (i,r) at A[i*ld + r]);
// otherwise it is contiguous along i (element (i,r) at A[r*ld + i]).
struct GemmDesc {
  const void* A; const void* B;
  int64_t I, J, R;
  int64_t lda, ldb;
  bool a_rc, b_rc;
  int wb;
};
// F1: C = Zsave [I][J] (storage type), bias [J], partial statistics part[tile][I] (float2).
void launch_generic_f1(int dt, const GemmDesc& g, const float* bias, void* Zsave, void* part, hipStream_t s);
// forward-product orientation with an optional bias and a ReLU or ReLU-mask epilogue (sibling operators)
void launch_generic_xwt(int dt, int kind, const GemmDesc& g, const float* bias, const void* aux, void* C, hipStream_t s);
// plain store: C [I][J] in the storage type
void launch_generic_store(int dt, const GemmDesc& g, void* C, hipStream_t s);
// plain store of the fp32 accumulators: C [I][J] float (bf16 storage; a partial sum for launch_fast_b4_reduce)
void launch_generic_store_f32(const GemmDesc& g, float* C, hipStream_t s);

// ---- row-wise / column-wise phases ------------------------------------------------------------
void launch_stats_finalize(const void* part, int tiles, int tile_w, int64_t M, int64_t N, float eps,
                           float* mean, float* rstd, hipStream_t s);
void launch_f2(int dt, int64_t M, int64_t N, const void* Zsave, const float* mean, const float* rstd,
               const float* gamma, const float* beta, void* Y, hipStream_t s);
// statistics and normalisation in one kernel (a wavefront per row); replaces FS + F2 when F1 emits no partials
bool f2_rows_supported(int dt, int64_t N);
void launch_f2_rows(int64_t M, int64_t N, float eps, const void* Zsave, const float* gamma, const float* beta, void* Y,
                    float* mean, float* rstd, hipStream_t s);
void launch_b1a(int dt, int64_t M, int64_t N, const void* dY, const void* Zsave, const float* gamma,
                const float* mean, const float* rstd, void* c12, hipStream_t s);
// ldz: pitch of dZ in elements (N, or N rounded up to the tile in the padded mode of the fast contractions)
void launch_b1b(int dt, int64_t M, int64_t N, int64_t ldz, int rows_per_group, int groups, const void* dY, const void* Zsave,
                const float* gamma, const float* mean, const float* rstd, const void* c12, void* dZ,
                void* colpart, hipStream_t s);
// fused single pass (row held in registers); returns false if this N is not supported by it
bool b1_fused_supported(int dt, int64_t N);
int b1_fused_groups(int dt, int64_t M, int64_t N);   // number of row groups it should be launched with (before capping at M)
// table: evaluate GELU from the LDS table, as the forward pass did (bf16, plan.f2_rows); else as the other kernels do
void launch_zero_cols_bf16(void* dZ, int64_t M, int64_t N, int64_t ldz, hipStream_t s);
// blocked: dZ is written as [M / 32][N / 32] blocks of 32 x 32 elements (bf16, M and N multiples of 32, ldz = N)
void launch_b1_fused(int dt, int64_t M, int64_t N, int64_t ldz, int groups, bool table, bool blocked, const void* dY,
                     const void* Zsave, const float* gamma, const float* mean, const float* rstd, void* dZ, void* colpart,
                     hipStream_t s);
void launch_b2(int dt, int64_t N, int groups, const void* colpart, float* dbeta, float* dgamma, float* db,
               hipStream_t s);
// bf16: the column sums (as launch_b2) and up to two sums of fp32 split-reduction partials
// (out[k][i] = bf16(sum over q < parts[k] of part[k][q * n[k] + i]); parts[k] = 0: none) in one launch
struct TailSums {
  const float* part[2];
  int parts[2];
  int64_t n[2];
  void* out[2];
  int blocks[2];          // filled in by launch_finish
  const float* colpart;   // [groups][3][N]
  int groups;
  int64_t N;
  float *dbeta, *dgamma, *db;
};
void launch_finish(TailSums j, hipStream_t s);

// ---- sibling operators' row-wise / element-wise kernels ------------------------------------------
void launch_layernorm(int dt, int64_t M, int64_t N, float eps, const void* A, const float* gamma, const float* beta,
                      void* Y, float* mean, float* rstd, hipStream_t s);
void launch_rmsnorm(int dt, int64_t M, int64_t N, float eps, const void* A, const float* weight, void* Y, hipStream_t s);
int colsum_groups(int64_t M);
// blocked: G is stored in 32 x 32 blocks (bf16; M, N multiples of 32)
void launch_colsum(int dt, int64_t M, int64_t N, const void* G, bool blocked, void* colpart, float* out, hipStream_t s);
void launch_silu_mul(int dt, int64_t n, const void* G, const void* U, void* H, hipStream_t s);

// ---- bf16 fast path -----------------------------------------------------------------------------
// F1 and B3 accept any M >= 128 (the last row tile may be partial); N, K as the tiles and the pipeline require.
bool fast_f1_supported(int64_t M, int64_t K, int64_t N);
bool fast_b3_supported(int64_t M, int64_t K, int64_t N);
// B4 reduces over M: the fast kernel takes the first fast_b4_rows(M) rows; the rest (< 128) is left to the caller
bool fast_b4_supported(int64_t M, int64_t K, int64_t N);
int64_t fast_b4_rows(int64_t M);
int fast_f1_stat_tile_w();
size_t fast_f1_tail_bytes(int64_t M, int64_t K);
// Wt: null, or the transposed weights [K][N] from launch_fast_transpose (N, K multiples of 64)
void launch_fast_transpose(int64_t N, int64_t K, const void* W, void* Wt, hipStream_t s);
void launch_fast_f1(int64_t M, int64_t K, int64_t N, const void* X, const void* W, const void* Wt, const float* bias,
                    void* Zsave, void* part, void* xtail, hipStream_t s);
// padded mode (N, K multiples of 8 but not both of 256): see gemm_bf16.hip
bool fast_padded_supported(int64_t M, int64_t K, int64_t N);
int64_t fast_pad_dim(int64_t n);
size_t fast_padded_tail_bytes(int64_t K);
int64_t fast_padded_b4_rows(int64_t M, int64_t K);
void launch_fast_pad_weights(int64_t K, int64_t N, const void* W, const float* bias, void* Wp, float* biasp, hipStream_t s);
void launch_fast_f1_padded(int64_t M, int64_t K, int64_t N, const void* X, const void* Wp, const float* biasp, void* Zsave,
                           void* part, void* xtail, hipStream_t s);
void launch_fast_b3_padded(int64_t M, int64_t K, int64_t N, const void* dZ, const void* Wp, void* dX, hipStream_t s);
void launch_fast_b4_padded(int64_t M, int64_t K, int64_t N, int split, const void* dZ, const void* X, void* dwpart,
                           hipStream_t s);
// sibling operators on the forward product's kernel (see gemm_bf16.hip); shapes as fast_f1_supported;
// Wt: null, or the transposed weights from launch_fast_transpose
constexpr int64_t kTransposeFromRows = 16384;   // batch size from which transposing the weights first pays
void launch_fast_xwt(int kind, int64_t M, int64_t K, int64_t N, const void* X, bool x_padded, const void* W,
                     const void* Wt, const float* bias, const void* aux, void* out, bool out_blocked, void* xtail,
                     hipStream_t s, bool x_blocked = false);   // x_blocked: X in 32 x 32 blocks (needs Wt, x_padded)
// gate and up products of the feed-forward block with the gated activation in the epilogue (see gemm_bf16.hip)
bool fast_gate_supported(int64_t M, int64_t D, int64_t H);
// Wcat: null, or the interleaved transposed weights [D][2H] from launch_fast_transpose_gate
void launch_fast_transpose_gate(int64_t H, int64_t D, const void* Wg, const void* Wu, void* Wcat, hipStream_t s);
void launch_fast_gate(int64_t M, int64_t D, int64_t H, const void* X, const void* Wg, const void* Wu, const void* Wcat,
                      void* Hout, bool out_blocked, void* xtail, hipStream_t s);
// dZ must have readable rows up to the next multiple of 256
// dz_blocked: dZ is stored in 32 x 32 blocks (launch_b1_fused with blocked = true; M, N multiples of 32)
void launch_fast_b3(int64_t M, int64_t K, int64_t N, const void* dZ, bool dz_blocked, const void* W, void* dX,
                    hipStream_t s);
int fast_b4_split(int64_t M, int64_t K, int64_t N);
void launch_fast_b4(int64_t M, int64_t K, int64_t N, int split, int extra, const void* dZ, bool dz_blocked, const void* X,
                    void* dW, void* dwpart, hipStream_t s);
void launch_fast_b4_reduce(int64_t K, int64_t N, int parts, const void* dwpart, void* dW, hipStream_t s);
// dX and dW in one launch where together they have at most a tile per compute unit; sa, sb: parts of the two reductions
bool fast_pair_plan(int64_t M, int64_t K, int64_t N, int* sa, int* sb);
void launch_fast_pair(int64_t M, int64_t K, int64_t N, int sa, int sb, const void* dZ, bool dz_blocked, const void* W,
                      const void* X, void* dX, void* dxpart, void* dW, void* dwpart, hipStream_t s);

}  // namespace fdl
