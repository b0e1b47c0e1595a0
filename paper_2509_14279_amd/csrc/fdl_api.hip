// C-ABI entry points of libfdl: argument validation, launch plan / workspace layout, and the sequence of
// kernel launches for the forward and backward pass of the fused dense-layer block.
#include "../../include/fdl.h"
#include "internal.h"

#include <cmath>
#include <cstdio>
#include <mutex>

namespace fdl {
namespace {

constexpr int64_t kMaxDim = (int64_t)1 << 24;       // per dimension
constexpr int64_t kMaxElems = (int64_t)1 << 40;     // per matrix

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

__global__ void zero_f32_kernel(float* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0.0f;
}
__global__ void zero_u16_kernel(unsigned short* p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

bool shape_ok(int64_t M, int64_t K, int64_t N) {
  if (M < 0 || K < 1 || N < 1) return false;
  if (M > kMaxDim || K > kMaxDim || N > kMaxDim) return false;
  if (M * N > kMaxElems || M * K > kMaxElems || N * K > kMaxElems) return false;
  return true;
}

bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Block tile of the generic kernel (as 16 x 16 blocks per wave tile side): 128 x 128 where that still gives every
// compute unit a tile, else 64 x 64.  fp32 storage always takes the small tile: its fp64 accumulators leave room for
// one workgroup per compute unit only at the large one, and with four the latencies of its register-staged loads are
// covered (measured: twice as fast on the forward contraction of the ragged fp32 configuration).
int pick_generic_wb(int dt, int64_t I, int64_t J) {
  if (dt == kF32) return 2;
  return (((I + 127) / 128) * ((J + 127) / 128) >= 256) ? 4 : 2;
}

thread_local bool t_failure_noted = false;

}  // namespace

void note_failure(const char* what, hipError_t e) {
  fprintf(stderr, "libfdl: %s failed: %s\n", what, hipGetErrorString(e));
  t_failure_noted = true;
}

bool device_info(DeviceInfo* out) {
  static std::mutex mu;
  static DeviceInfo cache[kMaxDevices];
  static bool have[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { note_failure("hipGetDevice", e); return false; }
  if (dev < 0 || dev >= kMaxDevices) { note_failure("device ordinal beyond the supported range", hipErrorInvalidDevice); return false; }
  std::lock_guard<std::mutex> lock(mu);
  if (!have[dev]) {
    int cus = 0, xcds = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess || cus < 1) { note_failure("hipDeviceGetAttribute(compute units)", e); return false; }
    // a runtime that does not know the attribute yet reports an error: every gfx950 part has 8 dies
    if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess || xcds < 1) {
      (void)hipGetLastError();
      xcds = 8;
    }
    if (cus % xcds != 0) xcds = 1;
    cache[dev].cus = cus; cache[dev].xcds = xcds;
    have[dev] = true;
  }
  *out = cache[dev];
  return true;
}

bool ensure_dynamic_lds(const void* kernel, int bytes, OnceFlags* flags) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) { note_failure("hipGetDevice", e); return false; }
  if (flags->done[dev].load(std::memory_order_acquire)) return true;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);   // idempotent: a race is harmless
  if (e != hipSuccess) { note_failure("hipFuncSetAttribute(dynamic LDS size)", e); return false; }
  flags->done[dev].store(1, std::memory_order_release);
  return true;
}

bool make_plan(int dt, int64_t M, int64_t K, int64_t N, Plan* p) {
  if (dt != kF32 && dt != kBF16) return false;
  if (!shape_ok(M, K, N)) return false;
  const size_t ts = dt == kF32 ? 4 : 2;   // storage element
  const size_t cs = dt == kF32 ? 8 : 4;   // arithmetic element
  Plan q = {};
  q.dt = dt; q.M = M; q.K = K; q.N = N;

  // ---- which contraction kernels run
  // bf16: the tuned kernel where N and K are multiples of the tile and the pipeline round (as they are), or - padded
  // mode - merely multiples of 8: the kernels then run on N and K rounded up to the tile, on a zero-padded copy of
  // the weights, and leave the surplus unstored.  Everything else takes the generic kernel.
  q.pad = dt == kBF16 && fast_padded_supported(M, K, N);
  const int64_t Np = q.pad ? fast_pad_dim(N) : N, Kp = q.pad ? fast_pad_dim(K) : K;
  q.ldz = Np;
  const int64_t Mp = M > 0 ? M : 1;
  auto pick_wb = [dt](int64_t I, int64_t J) { return pick_generic_wb(dt, I, J); };

  // ---- forward
  q.f1_fast = q.pad || (dt == kBF16 && fast_f1_supported(M, K, N));
  q.f2_rows = q.f1_fast && f2_rows_supported(dt, N);
  q.f1_wb = pick_wb(Mp, N);
  q.stat_tile_w = q.f1_fast ? fast_f1_stat_tile_w() : 16 * q.f1_wb;
  q.stat_tiles = (int)((N + q.stat_tile_w - 1) / q.stat_tile_w);
  size_t off = 0;
  q.off_part = off; off += align256(q.f2_rows ? 0 : (size_t)q.stat_tiles * Mp * 8);   // no partials where F2 takes the statistics
  q.off_xtail = off; off += align256(q.pad ? fast_padded_tail_bytes(K) : (q.f1_fast ? fast_f1_tail_bytes(M, K) : 0));
  q.off_wpad_f = off; off += align256(q.pad ? (size_t)Np * Kp * 2 : 0);
  q.off_bpad_f = off; off += align256(q.pad ? (size_t)Np * 4 : 0);
  // Large batches on the tuned kernel (tile-aligned N and K): the weights are transposed first, 4 N K bytes of traffic
  // against about 6 % of the contraction's time; that pays from roughly 10^4 rows, with a margin for the extra launch.
  q.fwd_bytes_plain = off;
  q.f1_wt = q.f1_fast && !q.pad && M >= kTransposeFromRows;
  q.off_wt = off; off += align256(q.f1_wt ? (size_t)N * K * 2 : 0);
  q.fwd_bytes = off;

  // ---- backward
  q.b1_fused = b1_fused_supported(dt, N);
  if (q.b1_fused) {
    const int64_t want = b1_fused_groups(dt, Mp, N);
    q.b1_groups = (int)(Mp < want ? Mp : want);
    q.b1_rows_per_group = 0;
  } else {
    int64_t rpg = (Mp + 1023) / 1024;
    if (rpg < 16) rpg = 16;
    q.b1_rows_per_group = (int)rpg;
    q.b1_groups = (int)((Mp + rpg - 1) / rpg);
  }
  q.b3_fast = q.pad || (dt == kBF16 && fast_b3_supported(M, K, N));
  q.b3_wb = pick_wb(Mp, K);
  q.b4_wb = pick_wb(N, K);
  if (q.pad) {
    q.b4_fast_rows = fast_padded_b4_rows(M, K);
    q.b4_fast = q.b4_fast_rows >= 128;
    if (!q.b4_fast) q.b4_fast_rows = 0;
  } else {
    q.b4_fast = dt == kBF16 && fast_b4_supported(M, K, N);
    q.b4_fast_rows = q.b4_fast ? fast_b4_rows(M) : 0;
  }
  q.b4_split = q.b4_fast ? fast_b4_split(q.b4_fast_rows, K, N) : 1;
  q.pair_sa = q.pair_sb = 1;
  q.pair = !q.pad && q.b3_fast && q.b4_fast && q.b4_fast_rows == M && fast_pair_plan(M, K, N, &q.pair_sa, &q.pair_sb);
  if (q.pair) q.b4_split = q.pair_sb;
  // dZ in 32 x 32 blocks where only the fused row kernel writes it and only the tuned kernels read it (no generic
  // kernel over the last rows, no padded pitch); the vector path of the row kernel needs N % 8 = 0, which the tiles imply
  // (the row kernel pays for it with about 8 % of its time where a row fills 1024 threads, dX gains about 9 %: not
  //  worth it when such rows meet a short K)
  q.dz_blocked = dt == kBF16 && q.b1_fused && !q.pad && q.b3_fast && q.b4_fast && q.b4_fast_rows == M && M % 32 == 0 &&
                 N % 32 == 0 && (K >= 1024 || N <= 4096);
  // fp32 partial sums of dW: the parts of a split reduction, one more for the rows the fast kernel leaves to the
  // generic one; in padded mode the fast kernel always writes partials
  int b4_parts = q.b4_split + (q.b4_fast && q.b4_fast_rows < M ? 1 : 0);
  if (q.pad && q.b4_fast && b4_parts < 2) b4_parts = 2;   // (a single part is still a partial: reduced into dW)
  off = 0;
  // dZ: the fast dX kernel reads whole 256-row tiles, so the buffer is rounded up (the surplus rows are never
  // written and never reach an output)
  q.off_dz = off; off += align256((size_t)((Mp + 255) / 256 * 256) * Np * ts);
  q.off_c12 = off; off += align256(q.b1_fused ? 0 : (size_t)2 * Mp * cs);
  q.off_colpart = off; off += align256((size_t)q.b1_groups * 3 * N * cs);
  q.off_dwpart = off; off += align256(b4_parts > 1 ? (size_t)b4_parts * N * K * 4 : 0);
  q.off_wpad_b = off; off += align256(q.pad ? (size_t)Np * Kp * 2 : 0);
  q.off_dxpart = off; off += align256(q.pair && q.pair_sa > 1 ? (size_t)q.pair_sa * M * K * 4 : 0);
  q.bwd_bytes = off;
  q.bytes = q.fwd_bytes > q.bwd_bytes ? q.fwd_bytes : q.bwd_bytes;
  *p = q;
  return true;
}

}  // namespace fdl

using namespace fdl;

extern "C" const char* fdl_status_string(fdl_status s) {
  switch (s) {
    case FDL_OK: return "FDL_OK";
    case FDL_ERR_NULL: return "FDL_ERR_NULL: a required pointer is NULL";
    case FDL_ERR_SHAPE: return "FDL_ERR_SHAPE: M, K or N out of the supported range";
    case FDL_ERR_DTYPE: return "FDL_ERR_DTYPE: unknown dtype";
    case FDL_ERR_EPS: return "FDL_ERR_EPS: eps must be finite and >= 0";
    case FDL_ERR_WORKSPACE: return "FDL_ERR_WORKSPACE: workspace missing or too small";
    case FDL_ERR_ALIGN: return "FDL_ERR_ALIGN: pointer not sufficiently aligned";
    case FDL_ERR_LAUNCH: return "FDL_ERR_LAUNCH: HIP reported a launch error";
  }
  return "unknown fdl_status";
}

extern "C" size_t fdl_workspace_bytes(fdl_dtype dt, int64_t M, int64_t K, int64_t N) {
  Plan p;
  if (!make_plan((int)dt, M, K, N, &p)) return 0;
  return p.bytes;
}

static fdl_status check_common(fdl_dtype dt, int64_t M, int64_t K, int64_t N, const void* workspace,
                               size_t workspace_bytes, Plan* p) {
  if (dt != FDL_F32 && dt != FDL_BF16) return FDL_ERR_DTYPE;
  if (!make_plan((int)dt, M, K, N, p)) return FDL_ERR_SHAPE;
  if (workspace == nullptr || workspace_bytes < p->bytes) return FDL_ERR_WORKSPACE;
  if (!aligned(workspace, 256)) return FDL_ERR_ALIGN;
  return FDL_OK;
}

// ---- optional per-phase event instrumentation
static hipEvent_t g_phase_events[2 * FDL_PHASE_COUNT];
static bool g_phase_events_on = false;

extern "C" fdl_status fdl_set_phase_events(void* const* events, int count) {
  if (events == nullptr) { g_phase_events_on = false; return FDL_OK; }
  if (count != 2 * FDL_PHASE_COUNT) return FDL_ERR_SHAPE;
  for (int i = 0; i < count; i++) {
    if (events[i] == nullptr) return FDL_ERR_NULL;
    g_phase_events[i] = static_cast<hipEvent_t>(events[i]);
  }
  g_phase_events_on = true;
  return FDL_OK;
}

namespace {
struct PhaseTimer {
  int phase; hipStream_t s;
  PhaseTimer(int p, hipStream_t st) : phase(p), s(st) {
    if (g_phase_events_on) (void)hipEventRecord(g_phase_events[2 * phase], s);
  }
  ~PhaseTimer() {
    if (g_phase_events_on) (void)hipEventRecord(g_phase_events[2 * phase + 1], s);
  }
};
}  // namespace

// The HIP "last error" is per-thread state shared with everything else the caller does on this thread (an
// allocator that probed and recovered from an out-of-memory condition leaves it set): it is cleared on entry so
// that only this call's launches are reported, and the reason of a failed launch goes to stderr.
static void clear_stale_error() { (void)hipGetLastError(); t_failure_noted = false; }
static fdl_status launch_status() {
  const hipError_t e = hipGetLastError();
  if (t_failure_noted) { t_failure_noted = false; return FDL_ERR_LAUNCH; }
  if (e == hipSuccess) return FDL_OK;
  fprintf(stderr, "libfdl: kernel launch failed: %s\n", hipGetErrorString(e));
  return FDL_ERR_LAUNCH;
}

// Validation shared by the forward entry points (everything except the scratch buffer).
static fdl_status check_forward_args(fdl_dtype dt, int64_t M, int64_t K, int64_t N, const void* X, const void* W,
                                     const float* b, const float* gamma, const float* beta, float eps, const void* Y,
                                     const void* Zsave, const float* mean, const float* rstd, Plan* p) {
  if (!X || !W || !b || !gamma || !beta || !Y || !Zsave || !mean || !rstd) return FDL_ERR_NULL;
  if (dt != FDL_F32 && dt != FDL_BF16) return FDL_ERR_DTYPE;
  if (!(eps >= 0.0f) || std::isinf(eps)) return FDL_ERR_EPS;
  if (!make_plan((int)dt, M, K, N, p)) return FDL_ERR_SHAPE;
  return FDL_OK;
}
static bool forward_args_aligned(const void* X, const void* W, const float* b, const float* gamma, const float* beta,
                                 const void* Y, const void* Zsave, const float* mean, const float* rstd) {
  return aligned(X, 16) && aligned(W, 16) && aligned(Y, 16) && aligned(Zsave, 16) && aligned(b, 16) &&
         aligned(gamma, 16) && aligned(beta, 16) && aligned(mean, 16) && aligned(rstd, 16);
}

// The launches of the forward pass; ws: at least p.fwd_bytes bytes of device scratch, 256-byte aligned.
static fdl_status forward_launches(const Plan& p, const void* X, const void* W, const float* b, const float* gamma,
                                   const float* beta, float eps, void* Y, void* Zsave, float* mean, float* rstd,
                                   char* ws, hipStream_t s) {
  const int64_t M = p.M, K = p.K, N = p.N;
  void* part = ws + p.off_part;
  {
    PhaseTimer t(FDL_PHASE_F1, s);
    if (p.pad) {
      void* Wp = ws + p.off_wpad_f;
      float* bp = reinterpret_cast<float*>(ws + p.off_bpad_f);
      launch_fast_pad_weights(K, N, W, b, Wp, bp, s);
      launch_fast_f1_padded(M, K, N, X, Wp, bp, Zsave, p.f2_rows ? nullptr : part, ws + p.off_xtail, s);
    } else if (p.f1_fast) {
      void* Wt = p.f1_wt ? ws + p.off_wt : nullptr;
      if (p.f1_wt) launch_fast_transpose(N, K, W, Wt, s);
      launch_fast_f1(M, K, N, X, W, Wt, b, Zsave, p.f2_rows ? nullptr : part, ws + p.off_xtail, s);
    } else {
      GemmDesc g = {X, W, M, N, K, K, K, true, true, p.f1_wb};
      launch_generic_f1(p.dt, g, b, Zsave, part, s);
    }
  }
  {
    PhaseTimer t(FDL_PHASE_FS, s);
    if (!p.f2_rows) launch_stats_finalize(part, p.stat_tiles, p.stat_tile_w, M, N, eps, mean, rstd, s);
  }
  {
    PhaseTimer t(FDL_PHASE_F2, s);
    if (p.f2_rows) launch_f2_rows(M, N, eps, Zsave, gamma, beta, Y, mean, rstd, s);
    else launch_f2(p.dt, M, N, Zsave, mean, rstd, gamma, beta, Y, s);
  }
  return launch_status();
}

extern "C" fdl_status fdl_forward(fdl_dtype dt, int64_t M, int64_t K, int64_t N, const void* X, const void* W,
                                  const float* b, const float* gamma, const float* beta, float eps, void* Y,
                                  void* Zsave, float* mean, float* rstd, void* workspace, size_t workspace_bytes,
                                  void* hip_stream) {
  Plan p;
  fdl_status st = check_forward_args(dt, M, K, N, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd, &p);
  if (st != FDL_OK) return st;
  st = check_common(dt, M, K, N, workspace, workspace_bytes, &p);
  if (st != FDL_OK) return st;
  if (!forward_args_aligned(X, W, b, gamma, beta, Y, Zsave, mean, rstd)) return FDL_ERR_ALIGN;
  if (M == 0) return FDL_OK;
  clear_stale_error();
  return forward_launches(p, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd, static_cast<char*>(workspace),
                          static_cast<hipStream_t>(hip_stream));
}

// ---- forward pass on the library's own scratch: no allocation, no workspace argument ----------------------------
// The scratch lives in device memory that belongs to the loaded code object: one copy per GPU, present from the
// moment the library is loaded on that GPU until the process ends.  In host code the array's name is only a handle;
// its device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[FDL_STATIC_SCRATCH_BYTES];

static char* static_scratch_address() {
  static std::mutex mu;
  static char* ptr[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) { note_failure("hipGetDevice", e); return nullptr; }
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* a = nullptr;
    e = hipGetSymbolAddress(&a, HIP_SYMBOL(scratch));
    if (e != hipSuccess || a == nullptr) { note_failure("hipGetSymbolAddress(static scratch)", e); return nullptr; }
    ptr[dev] = static_cast<char*>(a);
  }
  return ptr[dev];
}

extern "C" fdl_status fdl_forward_static(fdl_dtype dt, int64_t M, int64_t K, int64_t N, const void* X, const void* W,
                                         const float* b, const float* gamma, const float* beta, float eps, void* Y,
                                         void* Zsave, float* mean, float* rstd, void* hip_stream) {
  Plan p;
  const fdl_status st = check_forward_args(dt, M, K, N, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd, &p);
  if (st != FDL_OK) return st;
  if (p.fwd_bytes > (size_t)FDL_STATIC_SCRATCH_BYTES && p.f1_wt) {
    p.f1_wt = 0; p.fwd_bytes = p.fwd_bytes_plain;   // no room for the transposed weights: the kernel reads W as it is
  }
  if (p.fwd_bytes > (size_t)FDL_STATIC_SCRATCH_BYTES) return FDL_ERR_WORKSPACE;   // the problem needs more than the array holds
  if (!forward_args_aligned(X, W, b, gamma, beta, Y, Zsave, mean, rstd)) return FDL_ERR_ALIGN;
  if (M == 0) return FDL_OK;
  clear_stale_error();
  char* ws = static_scratch_address();
  if (ws == nullptr) return launch_status();
  // every scratch location a forward pass reads has been written earlier in the same pass (partial statistics
  // per row and column tile, the padded copy of X's last rows), so nothing has to be cleared between calls
  return forward_launches(p, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd, ws, static_cast<hipStream_t>(hip_stream));
}

extern "C" fdl_status fdl_backward(fdl_dtype dt, int64_t M, int64_t K, int64_t N, const void* dY, const void* X,
                                   const void* W, const float* gamma, const void* Zsave, const float* mean,
                                   const float* rstd, void* dX, void* dW, float* db, float* dgamma, float* dbeta,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!dY || !X || !W || !gamma || !Zsave || !mean || !rstd || !dX || !dW || !db || !dgamma || !dbeta)
    return FDL_ERR_NULL;
  Plan p;
  const fdl_status st = check_common(dt, M, K, N, workspace, workspace_bytes, &p);
  if (st != FDL_OK) return st;
  if (!aligned(dY, 16) || !aligned(X, 16) || !aligned(W, 16) || !aligned(Zsave, 16) || !aligned(dX, 16) ||
      !aligned(dW, 16) || !aligned(gamma, 16) || !aligned(mean, 16) || !aligned(rstd, 16) || !aligned(db, 16) ||
      !aligned(dgamma, 16) || !aligned(dbeta, 16))
    return FDL_ERR_ALIGN;
  clear_stale_error();
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (M == 0) {
    // no rows: every sum over rows is empty
    const int64_t nk = N * K;
    if (dt == FDL_F32) hipLaunchKernelGGL(zero_f32_kernel, dim3(256), dim3(256), 0, s, (float*)dW, nk);
    else hipLaunchKernelGGL(zero_u16_kernel, dim3(256), dim3(256), 0, s, (unsigned short*)dW, nk);
    hipLaunchKernelGGL(zero_f32_kernel, dim3(8), dim3(256), 0, s, db, N);
    hipLaunchKernelGGL(zero_f32_kernel, dim3(8), dim3(256), 0, s, dgamma, N);
    hipLaunchKernelGGL(zero_f32_kernel, dim3(8), dim3(256), 0, s, dbeta, N);
    return launch_status();
  }
  char* ws = static_cast<char*>(workspace);
  void* dZ = ws + p.off_dz;
  void* c12 = ws + p.off_c12;
  void* colpart = ws + p.off_colpart;

  {
    PhaseTimer t(FDL_PHASE_B1, s);
    if (p.b1_fused) {
      launch_b1_fused((int)dt, M, N, p.ldz, p.b1_groups, p.f2_rows != 0, p.dz_blocked != 0, dY, Zsave, gamma, mean, rstd, dZ,
                      colpart, s);
    } else {
      launch_b1a((int)dt, M, N, dY, Zsave, gamma, mean, rstd, c12, s);
      launch_b1b((int)dt, M, N, p.ldz, p.b1_rows_per_group, p.b1_groups, dY, Zsave, gamma, mean, rstd, c12, dZ, colpart, s);
    }
    if (p.pad) launch_zero_cols_bf16(dZ, M, N, p.ldz, s);   // the surplus columns enter the dX and dW contractions
  }
  // Where the contractions below leave split reductions behind (bf16 tuned path), their sums and the column sums
  // share one launch at the end of the pass; otherwise the column sums are finished here.
  const bool pair_sums = p.pair && (p.pair_sa > 1 || p.pair_sb > 1);
  const bool b4_sums = !p.pair && p.b4_fast && (p.pad || p.b4_split > 1 || p.b4_fast_rows < M);
  const bool tail = dt == FDL_BF16 && (pair_sums || b4_sums);
  TailSums tj = {};
  tj.colpart = static_cast<const float*>(colpart); tj.groups = p.b1_groups; tj.N = N;
  tj.dbeta = dbeta; tj.dgamma = dgamma; tj.db = db;
  auto sum_later = [&](int k, const void* part, int parts, int64_t n, void* out) {
    tj.part[k] = static_cast<const float*>(part); tj.parts[k] = parts; tj.n[k] = n; tj.out[k] = out;
  };
  {
    PhaseTimer t(FDL_PHASE_B2, s);
    if (!tail) launch_b2((int)dt, N, p.b1_groups, colpart, dbeta, dgamma, db, s);
  }
  {
    // B3: dX[M,K] = dZ[M,N] W[N,K]
    PhaseTimer t(FDL_PHASE_B3, s);
    if (p.pair) {
      // one launch for both contractions (B4 below only sums the partial sums of dW, where its reduction is split)
      launch_fast_pair(M, K, N, p.pair_sa, p.pair_sb, dZ, p.dz_blocked != 0, W, X, dX, ws + p.off_dxpart, dW,
                       ws + p.off_dwpart, s);
      if (p.pair_sa > 1) sum_later(0, ws + p.off_dxpart, p.pair_sa, M * K, dX);
    } else if (p.pad) {
      void* Wp = ws + p.off_wpad_b;
      launch_fast_pad_weights(K, N, W, nullptr, Wp, nullptr, s);
      launch_fast_b3_padded(M, K, N, dZ, Wp, dX, s);
    } else if (p.b3_fast) {
      launch_fast_b3(M, K, N, dZ, p.dz_blocked != 0, W, dX, s);
    } else {
      GemmDesc g = {dZ, W, M, K, N, p.ldz, K, true, false, p.b3_wb};
      launch_generic_store((int)dt, g, dX, s);
    }
  }
  {
    // B4: dW[N,K] = dZ^T[N,M] X[M,K]
    PhaseTimer t(FDL_PHASE_B4, s);
    if (p.pair) {
      if (p.pair_sb > 1) sum_later(1, ws + p.off_dwpart, p.pair_sb, N * K, dW);
    } else if (p.pad && p.b4_fast) {
      // padded mode: the fast kernel writes fp32 partials of the first b4_fast_rows rows; the generic kernel adds one
      // for the remaining rows (there is always at least one when K is not a multiple of the tile)
      const int64_t Mf = p.b4_fast_rows;
      float* dwpart = reinterpret_cast<float*>(ws + p.off_dwpart);
      launch_fast_b4_padded(Mf, K, N, p.b4_split, dZ, X, dwpart, s);
      int parts = p.b4_split;
      if (Mf < M) {
        const char* dZt = static_cast<const char*>(dZ) + (size_t)Mf * p.ldz * 2;
        const char* Xt = static_cast<const char*>(X) + (size_t)Mf * K * 2;
        GemmDesc g = {dZt, Xt, N, K, M - Mf, p.ldz, K, false, false, p.b4_wb};
        launch_generic_store_f32(g, dwpart + (size_t)parts * N * K, s);
        parts++;
      }
      sum_later(1, dwpart, parts, N * K, dW);
    } else if (p.b4_fast) {
      // the fast kernel reduces over the first b4_fast_rows rows (a whole number of pipeline rounds); the few rows
      // after them go through the generic kernel into one more fp32 partial sum
      const int64_t Mf = p.b4_fast_rows;
      const int extra = Mf < M ? 1 : 0;
      float* dwpart = reinterpret_cast<float*>(ws + p.off_dwpart);
      launch_fast_b4(Mf, K, N, p.b4_split, extra, dZ, p.dz_blocked != 0, X, dW, dwpart, s);
      if (extra) {
        const char* dZt = static_cast<const char*>(dZ) + (size_t)Mf * N * 2;
        const char* Xt = static_cast<const char*>(X) + (size_t)Mf * K * 2;
        GemmDesc g = {dZt, Xt, N, K, M - Mf, N, K, false, false, p.b4_wb};
        launch_generic_store_f32(g, dwpart + (size_t)p.b4_split * N * K, s);
      }
      if (p.b4_split + extra > 1) sum_later(1, dwpart, p.b4_split + extra, N * K, dW);
    } else {
      GemmDesc g = {dZ, X, N, K, M, p.ldz, K, false, false, p.b4_wb};
      launch_generic_store((int)dt, g, dW, s);
    }
    if (tail) launch_finish(tj, s);
  }
  return launch_status();
}


// =====================================================================================================================
// Forward-only variant and the sibling operators on the same kernels
// =====================================================================================================================

// ---- forward for inference: nothing is saved for a backward pass ---------------------------------------------------
// The pre-activation is written into Y and normalised there (the normalisation reads an element before it writes it),
// so no M x N scratch is needed: the workspace holds the row statistics, the partial statistics where the GEMM
// epilogue emits them, and the padded copy of X's last rows.
namespace {
struct InferencePlan { Plan p; size_t off_mean, off_rstd, bytes; };
bool make_inference_plan(int dt, int64_t M, int64_t K, int64_t N, InferencePlan* q) {
  if (!make_plan(dt, M, K, N, &q->p)) return false;
  const int64_t Mp = M > 0 ? M : 1;
  size_t off = q->p.fwd_bytes;
  q->off_mean = off; off += align256((size_t)Mp * 4);
  q->off_rstd = off; off += align256((size_t)Mp * 4);
  q->bytes = off;
  return true;
}
}  // namespace

extern "C" size_t fdl_forward_inference_workspace_bytes(fdl_dtype dt, int64_t M, int64_t K, int64_t N) {
  InferencePlan q;
  if (!make_inference_plan((int)dt, M, K, N, &q)) return 0;
  return q.bytes;
}

extern "C" fdl_status fdl_forward_inference(fdl_dtype dt, int64_t M, int64_t K, int64_t N, const void* X, const void* W,
                                            const float* b, const float* gamma, const float* beta, float eps, void* Y,
                                            void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!X || !W || !b || !gamma || !beta || !Y) return FDL_ERR_NULL;
  if (dt != FDL_F32 && dt != FDL_BF16) return FDL_ERR_DTYPE;
  if (!(eps >= 0.0f) || std::isinf(eps)) return FDL_ERR_EPS;
  InferencePlan q;
  if (!make_inference_plan((int)dt, M, K, N, &q)) return FDL_ERR_SHAPE;
  if (workspace == nullptr || workspace_bytes < q.bytes) return FDL_ERR_WORKSPACE;
  if (!aligned(workspace, 256)) return FDL_ERR_ALIGN;
  if (!aligned(X, 16) || !aligned(W, 16) || !aligned(Y, 16) || !aligned(b, 16) || !aligned(gamma, 16) || !aligned(beta, 16))
    return FDL_ERR_ALIGN;
  if (M == 0) return FDL_OK;
  clear_stale_error();
  char* ws = static_cast<char*>(workspace);
  return forward_launches(q.p, X, W, b, gamma, beta, eps, Y, /*Zsave=*/Y, reinterpret_cast<float*>(ws + q.off_mean),
                          reinterpret_cast<float*>(ws + q.off_rstd), ws, static_cast<hipStream_t>(hip_stream));
}

// ---- Linear + ReLU -------------------------------------------------------------------------------------------------
namespace {
// Workspace of the Linear+ReLU pair (one layout for both passes): the masked upstream gradient G [M][N] in the
// storage type with rows padded to whole tiles (the fast dX kernel reads whole tiles), the first-stage column
// partials of db, the fp32 partial sums of a split dW reduction, and the padded copy of X's last rows.
struct ReluPlan {
  int f1_fast, b3_fast, b4_fast, b4_split, f1_wb, b3_wb, b4_wb;
  int f1_wt;               // the forward product (and its recomputation) reads the weights from a transposed copy
  int g_blocked;           // the masked gradient G lives in 32 x 32 blocks (tuned kernels write and read all of it)
  int64_t b4_fast_rows;
  size_t off_g, off_colpart, off_dwpart, off_xtail, off_wt, bytes;
};
bool make_relu_plan(int dt, int64_t M, int64_t K, int64_t N, ReluPlan* q) {
  if (dt != kF32 && dt != kBF16) return false;
  if (!shape_ok(M, K, N)) return false;
  const size_t ts = dt == kF32 ? 4 : 2, cs = dt == kF32 ? 8 : 4;
  const int64_t Mp = M > 0 ? M : 1;
  auto pick_wb = [dt](int64_t I, int64_t J) { return pick_generic_wb(dt, I, J); };
  // the tuned kernels where the shape fits their tiles and pipeline rounds as it is; the generic kernel otherwise
  q->f1_fast = dt == kBF16 && fast_f1_supported(M, K, N);
  q->b3_fast = dt == kBF16 && fast_b3_supported(M, K, N);
  q->b4_fast = dt == kBF16 && fast_b4_supported(M, K, N);
  q->b4_fast_rows = q->b4_fast ? fast_b4_rows(M) : 0;
  q->b4_split = q->b4_fast ? fast_b4_split(q->b4_fast_rows, K, N) : 1;
  q->f1_wb = pick_wb(Mp, N); q->b3_wb = pick_wb(Mp, K); q->b4_wb = pick_wb(N, K);
  const int b4_parts = q->b4_split + (q->b4_fast && q->b4_fast_rows < M ? 1 : 0);
  size_t off = 0;
  q->off_g = off; off += align256((size_t)((Mp + 255) / 256 * 256) * N * ts);
  q->off_colpart = off; off += align256((size_t)colsum_groups(Mp) * N * cs);
  q->off_dwpart = off; off += align256(b4_parts > 1 ? (size_t)b4_parts * N * K * 4 : 0);
  q->off_xtail = off; off += align256(q->f1_fast ? fast_f1_tail_bytes(M, K) : 0);
  q->f1_wt = q->f1_fast && M >= kTransposeFromRows;
  q->off_wt = off; off += align256(q->f1_wt ? (size_t)N * K * 2 : 0);
  q->g_blocked = q->f1_fast && q->b3_fast && q->b4_fast && q->b4_fast_rows == M && M % 32 == 0 && N % 32 == 0;
  q->bytes = off;
  return true;
}
fdl_status check_ws(const void* workspace, size_t have, size_t need) {
  if (workspace == nullptr || have < need) return FDL_ERR_WORKSPACE;
  if (!aligned(workspace, 256)) return FDL_ERR_ALIGN;
  return FDL_OK;
}
}  // namespace

extern "C" size_t fdl_linear_relu_workspace_bytes(fdl_dtype dt, int64_t M, int64_t K, int64_t N) {
  ReluPlan q;
  if (!make_relu_plan((int)dt, M, K, N, &q)) return 0;
  return q.bytes;
}

extern "C" fdl_status fdl_linear_relu_forward(fdl_dtype dt, int64_t M, int64_t K, int64_t N, const void* X, const void* W,
                                              const float* b, void* Y, void* workspace, size_t workspace_bytes,
                                              void* hip_stream) {
  if (!X || !W || !b || !Y) return FDL_ERR_NULL;
  if (dt != FDL_F32 && dt != FDL_BF16) return FDL_ERR_DTYPE;
  ReluPlan q;
  if (!make_relu_plan((int)dt, M, K, N, &q)) return FDL_ERR_SHAPE;
  const fdl_status st = check_ws(workspace, workspace_bytes, q.bytes);
  if (st != FDL_OK) return st;
  if (!aligned(X, 16) || !aligned(W, 16) || !aligned(Y, 16) || !aligned(b, 16)) return FDL_ERR_ALIGN;
  if (M == 0) return FDL_OK;
  clear_stale_error();
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  if (q.f1_fast) {
    void* Wt = q.f1_wt ? ws + q.off_wt : nullptr;
    if (q.f1_wt) launch_fast_transpose(N, K, W, Wt, s);
    launch_fast_xwt(1, M, K, N, X, false, W, Wt, b, nullptr, Y, false, ws + q.off_xtail, s);
  } else {
    GemmDesc g = {X, W, M, N, K, K, K, true, true, q.f1_wb};
    launch_generic_xwt((int)dt, 1, g, b, nullptr, Y, s);
  }
  return launch_status();
}

extern "C" fdl_status fdl_linear_relu_backward(fdl_dtype dt, int64_t M, int64_t K, int64_t N, const void* dY, const void* X,
                                               const void* W, const float* b, void* dX, void* dW, float* db,
                                               void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!dY || !X || !W || !b || !dX || !dW || !db) return FDL_ERR_NULL;
  if (dt != FDL_F32 && dt != FDL_BF16) return FDL_ERR_DTYPE;
  ReluPlan q;
  if (!make_relu_plan((int)dt, M, K, N, &q)) return FDL_ERR_SHAPE;
  const fdl_status st = check_ws(workspace, workspace_bytes, q.bytes);
  if (st != FDL_OK) return st;
  if (!aligned(dY, 16) || !aligned(X, 16) || !aligned(W, 16) || !aligned(b, 16) || !aligned(dX, 16) || !aligned(dW, 16) ||
      !aligned(db, 16))
    return FDL_ERR_ALIGN;
  clear_stale_error();
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const ReluPlan& p = q;
  if (M == 0) {
    const int64_t nk = N * K;
    if (dt == FDL_F32) hipLaunchKernelGGL(zero_f32_kernel, dim3(256), dim3(256), 0, s, (float*)dW, nk);
    else hipLaunchKernelGGL(zero_u16_kernel, dim3(256), dim3(256), 0, s, (unsigned short*)dW, nk);
    hipLaunchKernelGGL(zero_f32_kernel, dim3(8), dim3(256), 0, s, db, N);
    return launch_status();
  }
  char* ws = static_cast<char*>(workspace);
  void* G = ws + q.off_g;
  void* colpart = ws + q.off_colpart;
  // G = dY where X W^T + b > 0: the pre-activation is recomputed and never stored
  if (p.f1_fast) {
    void* Wt = p.f1_wt ? ws + q.off_wt : nullptr;
    if (p.f1_wt) launch_fast_transpose(N, K, W, Wt, s);
    launch_fast_xwt(2, M, K, N, X, false, W, Wt, b, dY, G, p.g_blocked != 0, ws + q.off_xtail, s);
  } else {
    GemmDesc g = {X, W, M, N, K, K, K, true, true, p.f1_wb};
    launch_generic_xwt((int)dt, 2, g, b, dY, G, s);
  }
  launch_colsum((int)dt, M, N, G, p.g_blocked != 0, colpart, db, s);
  if (p.b3_fast) {
    launch_fast_b3(M, K, N, G, p.g_blocked != 0, W, dX, s);
  } else {
    GemmDesc g = {G, W, M, K, N, N, K, true, false, p.b3_wb};
    launch_generic_store((int)dt, g, dX, s);
  }
  if (p.b4_fast) {
    const int64_t Mf = p.b4_fast_rows;
    const int extra = Mf < M ? 1 : 0;
    float* dwpart = reinterpret_cast<float*>(ws + q.off_dwpart);
    launch_fast_b4(Mf, K, N, p.b4_split, extra, G, p.g_blocked != 0, X, dW, dwpart, s);
    if (extra) {
      const char* Gt = static_cast<const char*>(G) + (size_t)Mf * N * 2;
      const char* Xt = static_cast<const char*>(X) + (size_t)Mf * K * 2;
      GemmDesc g = {Gt, Xt, N, K, M - Mf, N, K, false, false, p.b4_wb};
      launch_generic_store_f32(g, dwpart + (size_t)p.b4_split * N * K, s);
    }
    if (p.b4_split + extra > 1) launch_fast_b4_reduce(K, N, p.b4_split + extra, dwpart, dW, s);
  } else {
    GemmDesc g = {G, X, N, K, M, N, K, false, false, p.b4_wb};
    launch_generic_store((int)dt, g, dW, s);
  }
  return launch_status();
}

// ---- LayerNorm and RMSNorm forward ---------------------------------------------------------------------------------
static bool norm_shape_ok(int64_t M, int64_t N) {
  return M >= 0 && N >= 1 && M <= kMaxDim && N <= kMaxDim && M * N <= kMaxElems;
}

extern "C" fdl_status fdl_layernorm_forward(fdl_dtype dt, int64_t M, int64_t N, const void* A, const float* gamma,
                                            const float* beta, float eps, void* Y, float* mean, float* rstd,
                                            void* hip_stream) {
  if (!A || !gamma || !beta || !Y || !mean || !rstd) return FDL_ERR_NULL;
  if (dt != FDL_F32 && dt != FDL_BF16) return FDL_ERR_DTYPE;
  if (!(eps >= 0.0f) || std::isinf(eps)) return FDL_ERR_EPS;
  if (!norm_shape_ok(M, N)) return FDL_ERR_SHAPE;
  if (!aligned(A, 16) || !aligned(Y, 16) || !aligned(gamma, 16) || !aligned(beta, 16) || !aligned(mean, 16) || !aligned(rstd, 16))
    return FDL_ERR_ALIGN;
  if (M == 0) return FDL_OK;
  clear_stale_error();
  launch_layernorm((int)dt, M, N, eps, A, gamma, beta, Y, mean, rstd, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

extern "C" fdl_status fdl_rmsnorm_forward(fdl_dtype dt, int64_t M, int64_t N, const void* A, const float* weight, float eps,
                                          void* Y, void* hip_stream) {
  if (!A || !weight || !Y) return FDL_ERR_NULL;
  if (dt != FDL_F32 && dt != FDL_BF16) return FDL_ERR_DTYPE;
  if (!(eps >= 0.0f) || std::isinf(eps)) return FDL_ERR_EPS;
  if (!norm_shape_ok(M, N)) return FDL_ERR_SHAPE;
  if (!aligned(A, 16) || !aligned(Y, 16) || !aligned(weight, 16)) return FDL_ERR_ALIGN;
  if (M == 0) return FDL_OK;
  clear_stale_error();
  launch_rmsnorm((int)dt, M, N, eps, A, weight, Y, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

// ---- Llama feed-forward block, forward -----------------------------------------------------------------------------
namespace {
// Workspace: G and U [Mpad][H] in the storage type (the activation overwrites G; rows padded to whole tiles so that the
// down projection's fast kernel may read a partial last row tile; U only where the two products are separate kernels),
// then the padded copy of X's last rows.
struct FfnPlan {
  int gate_fused;          // 1: one kernel forms both products and the gated activation (no M x H round trip)
  int up_fast, down_fast, up_wb, down_wb;
  int down_wt;             // the down projection reads its weights from a transposed copy
  int gate_wt;             // the fused gate/up kernel reads both weight matrices from one interleaved transposed copy
  int g_blocked;           // the gated activation passes from the fused kernel to the down projection in 32 x 32 blocks
  size_t off_g, off_u, off_xtail, off_wt, off_wcat, bytes;
};
bool make_ffn_plan(int dt, int64_t M, int64_t D, int64_t H, FfnPlan* q) {
  if (dt != kF32 && dt != kBF16) return false;
  if (M < 0 || D < 1 || H < 1 || M > kMaxDim || D > kMaxDim || H > kMaxDim) return false;
  if (M * H > kMaxElems || M * D > kMaxElems || H * D > kMaxElems) return false;
  const size_t ts = dt == kF32 ? 4 : 2;
  const int64_t Mp = M > 0 ? M : 1;
  auto pick_wb = [dt](int64_t I, int64_t J) { return pick_generic_wb(dt, I, J); };
  q->gate_fused = dt == kBF16 && fast_gate_supported(M, D, H);
  q->up_fast = dt == kBF16 && fast_f1_supported(M, D, H);      // [M,D] x [H,D]^T
  q->down_fast = dt == kBF16 && fast_f1_supported(M, H, D);    // [M,H] x [D,H]^T
  q->up_wb = pick_wb(Mp, H);
  q->down_wb = pick_wb(Mp, D);
  size_t off = 0;
  const size_t mh = align256((size_t)((Mp + 255) / 256 * 256) * H * ts);
  q->off_g = off; off += mh;
  q->off_u = off; off += q->gate_fused ? 0 : mh;    // the fused kernel never materialises the up product
  q->off_xtail = off; off += align256((q->up_fast || q->gate_fused) ? fast_f1_tail_bytes(M, D) : 0);
  q->down_wt = q->down_fast && M >= kTransposeFromRows;
  q->off_wt = off; off += align256(q->down_wt ? (size_t)D * H * 2 : 0);
  q->gate_wt = q->gate_fused && M >= kTransposeFromRows && H % 64 == 0 && D % 64 == 0;
  q->off_wcat = off; off += align256(q->gate_wt ? (size_t)2 * D * H * 2 : 0);
  q->g_blocked = q->gate_fused && q->down_wt && H % 32 == 0;
  q->bytes = off;
  return true;
}
}  // namespace

extern "C" size_t fdl_llama_ffn_workspace_bytes(fdl_dtype dt, int64_t M, int64_t D, int64_t H) {
  FfnPlan q;
  if (!make_ffn_plan((int)dt, M, D, H, &q)) return 0;
  return q.bytes;
}

extern "C" fdl_status fdl_llama_ffn_forward(fdl_dtype dt, int64_t M, int64_t D, int64_t H, const void* X, const void* Wg,
                                            const void* Wu, const void* Wd, void* Y, void* workspace,
                                            size_t workspace_bytes, void* hip_stream) {
  if (!X || !Wg || !Wu || !Wd || !Y) return FDL_ERR_NULL;
  if (dt != FDL_F32 && dt != FDL_BF16) return FDL_ERR_DTYPE;
  FfnPlan q;
  if (!make_ffn_plan((int)dt, M, D, H, &q)) return FDL_ERR_SHAPE;
  const fdl_status st = check_ws(workspace, workspace_bytes, q.bytes);
  if (st != FDL_OK) return st;
  if (!aligned(X, 16) || !aligned(Wg, 16) || !aligned(Wu, 16) || !aligned(Wd, 16) || !aligned(Y, 16)) return FDL_ERR_ALIGN;
  if (M == 0) return FDL_OK;
  clear_stale_error();
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  void* G = ws + q.off_g;
  void* U = ws + q.off_u;
  if (q.gate_fused) {
    void* Wcat = q.gate_wt ? ws + q.off_wcat : nullptr;
    if (q.gate_wt) launch_fast_transpose_gate(H, D, Wg, Wu, Wcat, s);
    launch_fast_gate(M, D, H, X, Wg, Wu, Wcat, G, q.g_blocked != 0, ws + q.off_xtail, s);
  } else if (q.up_fast) {
    launch_fast_xwt(0, M, D, H, X, false, Wg, nullptr, nullptr, nullptr, G, false, ws + q.off_xtail, s);
    launch_fast_xwt(0, M, D, H, X, false, Wu, nullptr, nullptr, nullptr, U, false, ws + q.off_xtail, s);
  } else {
    GemmDesc g = {X, Wg, M, H, D, D, D, true, true, q.up_wb};
    launch_generic_xwt((int)dt, 0, g, nullptr, nullptr, G, s);
    g.B = Wu;
    launch_generic_xwt((int)dt, 0, g, nullptr, nullptr, U, s);
  }
  if (!q.gate_fused) launch_silu_mul((int)dt, M * H, G, U, G, s);
  if (q.down_fast) {
    void* Wt = q.down_wt ? ws + q.off_wt : nullptr;
    if (q.down_wt) launch_fast_transpose(D, H, Wd, Wt, s);
    launch_fast_xwt(0, M, H, D, G, /*x_padded=*/true, Wd, Wt, nullptr, nullptr, Y, false, nullptr, s, q.g_blocked != 0);
  } else {
    GemmDesc g = {G, Wd, M, D, H, H, H, true, true, q.down_wb};
    launch_generic_xwt((int)dt, 0, g, nullptr, nullptr, Y, s);
  }
  return launch_status();
}
