// Measured ceilings of one MI355X (gfx950) for the roofline report: what the matrix cores, the HBM interface and
// the LDS deliver to the simplest possible kernels.  Benchmark support only: built into its own shared object
// (libfdl_ceilings.so), never linked into libfdl.so.  C ABI; every call enqueues kernels on the given stream.
//
//   fdlc_mfma_bf16      register-resident v_mfma_f32_32x32x16_bf16 loop, one or two waves per SIMD on every CU
//   fdlc_mfma_f64       the same for v_mfma_f64_16x16x4_f64 (the fp32-storage path's instruction)
//   fdlc_stream_*       read-only / write-only / copy / two-reads-one-write over large buffers, 16 bytes per lane,
//                       non-temporal
//   fdlc_lds_probe      one LDS read instruction in a tight loop with a chosen lane -> address pattern, timed with the
//                       shader clock (cycles per instruction) - the patterns of the GEMM kernel's fragment reads next
//                       to a linear (trivially conflict-free) and a same-bank (worst case) pattern
#include <hip/hip_runtime.h>
#include <stdint.h>

#define FDLC_API extern "C" __attribute__((visibility("default")))

namespace {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// a bf16 value in (-2, 2) with a varied bit pattern (operand toggling matters for power)
__device__ __forceinline__ bf16_t pseudo(uint32_t i) {
  const uint32_t h = mix(i);
  const float v = ((float)(h & 0xffff) / 32768.0f - 1.0f) * 2.0f;
  return (bf16_t)v;
}

// ---------------------------------------------------------------------------------------------- MFMA
// 4 x NB independent accumulator blocks, 4 + NB operand fragments, all in registers.  NB = 4 with one wave per SIMD
// is the GEMM kernel's own shape (256 accumulator registers per lane); NB = 2 with two waves per SIMD halves both.
template <int NB, int WAVES>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(WAVES / 4, WAVES / 4)))
void mfma_bf16_kernel(int iters, float* out) {
  bf16x8 a[4], b[NB];
  for (int i = 0; i < 4; i++)
    for (int e = 0; e < 8; e++) a[i][e] = pseudo((threadIdx.x * 4 + i) * 8 + e);
  for (int j = 0; j < NB; j++)
    for (int e = 0; e < 8; e++) b[j][e] = pseudo(0x10000u + (threadIdx.x * 4 + j) * 8 + e);
  f32x16 acc[4][NB];
  for (int i = 0; i < 4; i++)
    for (int j = 0; j < NB; j++)
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.0f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < NB; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; i++) asm volatile("" : "+v"(a[i]));   // the operands stay opaque: nothing is hoisted or folded
  }
  float s = 0.0f;
  for (int i = 0; i < 4; i++)
    for (int j = 0; j < NB; j++)
      for (int r = 0; r < 16; r++) s += acc[i][j][r];
  if (s == 123.456f) out[0] = s;   // keeps the loop alive; practically never true
}

// The fp32-storage path's instruction: v_mfma_f64_16x16x4_f64, 4 x 4 independent accumulator blocks per wave (the
// generic kernel has 2 x 2 with four reduction steps each), one wave per SIMD.
__global__ __launch_bounds__(256) void mfma_f64_kernel(int iters, float* out) {
  typedef __attribute__((ext_vector_type(4))) double f64x4;
  double a[4], b[4];
  for (int i = 0; i < 4; i++) { a[i] = (double)(float)pseudo(threadIdx.x * 4 + i); b[i] = (double)(float)pseudo(0x10000u + threadIdx.x * 4 + i); }
  f64x4 acc[4][4];
  for (int i = 0; i < 4; i++)
    for (int j = 0; j < 4; j++)
      for (int r = 0; r < 4; r++) acc[i][j][r] = 0.0;
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++) asm volatile("" : "+a"(acc[i][j]));
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; i++) asm volatile("" : "+v"(a[i]));
    // the accumulators stay in AGPRs from one round to the next (left to itself the compiler moves all 128 registers
    // to VGPRs and back in every round, and the loop then measures those moves: 36 instead of 77 TFLOP/s)
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++) asm volatile("" : "+a"(acc[i][j]));
  }
  double s = 0.0;
  for (int i = 0; i < 4; i++)
    for (int j = 0; j < 4; j++)
      for (int r = 0; r < 4; r++) s += acc[i][j][r];
  if (s == 123.456) out[0] = (float)s;
}

// ---------------------------------------------------------------------------------------------- streaming
// Each workgroup of 1024 threads walks contiguous chunks of 1024 x U vectors of 16 bytes (U = 16: 256 KB) with grid
// stride; all loads of a chunk are issued before its first store.  n16: number of 16-byte vectors.
constexpr int kStreamU = 16;
constexpr int kStreamThreads = 1024;
__global__ __launch_bounds__(kStreamThreads) void stream_read_kernel(const u32x4* __restrict__ src, int64_t n16, uint32_t* sink) {
  const int64_t chunk = (int64_t)kStreamThreads * kStreamU;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int64_t base = (int64_t)blockIdx.x * chunk; base < n16; base += (int64_t)gridDim.x * chunk) {
#pragma unroll
    for (int u = 0; u < kStreamU; u++) {
      const int64_t i = base + (int64_t)u * kStreamThreads + threadIdx.x;
      if (i < n16) acc ^= __builtin_nontemporal_load(src + i);
    }
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = acc[0];
}
__global__ __launch_bounds__(kStreamThreads) void stream_write_kernel(u32x4* __restrict__ dst, int64_t n16) {
  const int64_t chunk = (int64_t)kStreamThreads * kStreamU;
  const u32x4 v = {threadIdx.x, blockIdx.x, 0x3f803f80u, 0xbf80bf80u};
  for (int64_t base = (int64_t)blockIdx.x * chunk; base < n16; base += (int64_t)gridDim.x * chunk) {
#pragma unroll
    for (int u = 0; u < kStreamU; u++) {
      const int64_t i = base + (int64_t)u * kStreamThreads + threadIdx.x;
      if (i < n16) __builtin_nontemporal_store(v, dst + i);
    }
  }
}
__global__ __launch_bounds__(kStreamThreads) void stream_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, int64_t n16) {
  const int64_t chunk = (int64_t)kStreamThreads * kStreamU;
  for (int64_t base = (int64_t)blockIdx.x * chunk; base < n16; base += (int64_t)gridDim.x * chunk) {
    u32x4 v[kStreamU];
#pragma unroll
    for (int u = 0; u < kStreamU; u++) {
      const int64_t i = base + (int64_t)u * kStreamThreads + threadIdx.x;
      if (i < n16) v[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < kStreamU; u++) {
      const int64_t i = base + (int64_t)u * kStreamThreads + threadIdx.x;
      if (i < n16) __builtin_nontemporal_store(v[u], dst + i);
    }
  }
}
// two reads per write: the mix of the backward row pass (reads dY and Zsave, writes dZ)
__global__ __launch_bounds__(kStreamThreads) void stream_mix21_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ a,
                                                                      const u32x4* __restrict__ b, int64_t n16) {
  constexpr int U = kStreamU / 2;
  const int64_t chunk = (int64_t)kStreamThreads * U;
  for (int64_t base = (int64_t)blockIdx.x * chunk; base < n16; base += (int64_t)gridDim.x * chunk) {
    u32x4 va[U], vb[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int64_t i = base + (int64_t)u * kStreamThreads + threadIdx.x;
      if (i < n16) { va[u] = __builtin_nontemporal_load(a + i); vb[u] = __builtin_nontemporal_load(b + i); }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int64_t i = base + (int64_t)u * kStreamThreads + threadIdx.x;
      if (i < n16) __builtin_nontemporal_store(va[u] ^ vb[u], dst + i);
    }
  }
}

// ---------------------------------------------------------------------------------------------- LDS probes
// Lane -> byte offset inside a 64 KB LDS tile for each pattern (the formulas of the GEMM kernel's fragment reads
// are restated here on purpose: this file shares no code with the library).
// (7-9: the swizzles the GEMM kernel used before, laid out for 32 banks - kept as the reference for what a two-way
// conflict costs and for what the bank-conflict counter reads on it.)
enum { LDS_B128_LINEAR = 0, LDS_B128_GEMM_BK64 = 1, LDS_B128_GEMM_BK32 = 2, LDS_TR16_GEMM = 3, LDS_B128_SAME_BANK = 4,
       LDS_B64_LINEAR = 5, LDS_B32_LINEAR = 6, LDS_B128_OLD_BK64 = 7, LDS_B128_OLD_BK32 = 8, LDS_TR16_OLD = 9,
       LDS_PATTERNS = 10 };

template <int PAT> __device__ __forceinline__ uint32_t lds_offset(int lane, int step) {
  if (PAT == LDS_B128_LINEAR) return (uint32_t)(lane * 16 + step * 1024);
  if (PAT == LDS_B128_GEMM_BK64 || PAT == LDS_B128_OLD_BK64) {
    // rows of 128 B; 16-byte chunk c of row r in slot c ^ ((r >> 1) & 7) (before: c ^ (r & 7)); sub-slice kk = step & 3
    const int row = (lane & 31) + 32 * (step >> 2), kk = step & 3, c = (kk << 1) | (lane >> 5);
    const int sw = PAT == LDS_B128_GEMM_BK64 ? (row >> 1) & 7 : row & 7;
    return (uint32_t)(row * 128 + (((c ^ sw) & 7) << 4));
  }
  if (PAT == LDS_B128_GEMM_BK32 || PAT == LDS_B128_OLD_BK32) {
    // rows of 64 B; chunk c of row r in slot c ^ ((r >> 2) & 3) (before: c ^ ((r >> 1) & 3))
    const int row = (lane & 31) + 32 * (step >> 1), kk = step & 1, c = (kk << 1) | (lane >> 5);
    const int sw = PAT == LDS_B128_GEMM_BK32 ? (row >> 2) & 3 : (row >> 1) & 3;
    return (uint32_t)(row * 64 + (((c ^ sw) & 3) << 4));
  }
  if (PAT == LDS_TR16_GEMM || PAT == LDS_TR16_OLD) {
    // r-major tile [r][32 chunks of 16 B], chunk c of r-row w in slot c ^ ((w & 3) << 2) (before: << 1)
    const int G = lane >> 4, p = lane & 15, r = 8 * (G >> 1) + (p >> 2);
    const int c = (step & 3) * 4 + 2 * (G & 1) + ((p & 3) >> 1);
    const int sw = (p >> 2) << (PAT == LDS_TR16_GEMM ? 2 : 1);
    return (uint32_t)((r + 16 * (step >> 2)) * 512 + ((c ^ sw) * 16) + (p & 1) * 8);
  }
  if (PAT == LDS_B128_SAME_BANK) return (uint32_t)(lane * 512 + step * 16);   // every lane on the same banks
  if (PAT == LDS_B64_LINEAR) return (uint32_t)(lane * 8 + step * 512);
  return (uint32_t)(lane * 4 + step * 256);
}

// out[2 * blockIdx.x] = shader-clock cycles of the timed loop (wave 0), out[2 * blockIdx.x + 1] = 100 MHz ticks
template <int PAT>
__global__ __launch_bounds__(256) void lds_probe_kernel(int iters, int64_t* out) {
  __shared__ __attribute__((aligned(1024))) uint32_t tile[16384];   // 64 KB
  for (int i = threadIdx.x; i < 16384; i += 256) tile[i] = mix(i);
  __syncthreads();
  const int lane = threadIdx.x & 63;
  typedef __attribute__((address_space(3))) uint32_t lds_u32;
  const uint32_t base = (uint32_t)(uintptr_t)(const lds_u32*)tile;   // LDS byte address of the tile
  uint32_t off[8];
#pragma unroll
  for (int s = 0; s < 8; s++) off[s] = base + (lds_offset<PAT>(lane, s) & 0xffffu);
  // The reads are issued from inline assembly so that the compiler can neither narrow nor merge them, and their
  // results are consumed by an empty statement: the loop holds 8 LDS reads, one wait and the loop control.
  uint32_t keep = 0;
  const int64_t c0 = (int64_t)clock64(), t0 = (int64_t)wall_clock64();
  for (int it = 0; it < iters; it++) {
    if (PAT == LDS_TR16_GEMM || PAT == LDS_TR16_OLD || PAT == LDS_B64_LINEAR) {
      u32x2 v[8];
#pragma unroll
      for (int s = 0; s < 8; s++) {
        if (PAT != LDS_B64_LINEAR) asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v[s]) : "v"(off[s]));
        else asm volatile("ds_read_b64 %0, %1" : "=v"(v[s]) : "v"(off[s]));
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("" :: "v"(v[s]));
      if (it == iters - 1) keep = v[0][0];
    } else if (PAT == LDS_B32_LINEAR) {
      uint32_t v[8];
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("ds_read_b32 %0, %1" : "=v"(v[s]) : "v"(off[s]));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("" :: "v"(v[s]));
      if (it == iters - 1) keep = v[0];
    } else {
      u32x4 v[8];
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("ds_read_b128 %0, %1" : "=v"(v[s]) : "v"(off[s]));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("" :: "v"(v[s]));
      if (it == iters - 1) keep = v[0][0];
    }
  }
  const int64_t c1 = (int64_t)clock64(), t1 = (int64_t)wall_clock64();
  if (threadIdx.x == 0) { out[2 * blockIdx.x] = c1 - c0; out[2 * blockIdx.x + 1] = t1 - t0; }
  if (keep == 0x12345678u && tile[threadIdx.x] == 77u) out[0] = 0;
}

// The same loop with the lane -> byte offset table read from memory (offsets[8][64], each < 65536 and a multiple of
// the access width): lets the host time any pattern without a rebuild.  KIND: 16 = ds_read_b128, 8 = ds_read_b64,
// 4 = ds_read_b32, -8 = ds_read_b64_tr_b16.
template <int KIND>
__global__ __launch_bounds__(256) void lds_probe_table_kernel(const uint32_t* __restrict__ offsets, int iters, int64_t* out) {
  __shared__ __attribute__((aligned(1024))) uint32_t tile[16384];   // 64 KB
  for (int i = threadIdx.x; i < 16384; i += 256) tile[i] = mix(i);
  __syncthreads();
  const int lane = threadIdx.x & 63;
  typedef __attribute__((address_space(3))) uint32_t lds_u32;
  const uint32_t base = (uint32_t)(uintptr_t)(const lds_u32*)tile;
  constexpr uint32_t kMask = KIND == 16 ? 0xfff0u : (KIND == 4 ? 0xfffcu : 0xfff8u);
  uint32_t off[8];
#pragma unroll
  for (int s = 0; s < 8; s++) off[s] = base + (offsets[s * 64 + lane] & kMask);
  uint32_t keep = 0;
  const int64_t c0 = (int64_t)clock64(), t0 = (int64_t)wall_clock64();
  for (int it = 0; it < iters; it++) {
    if (KIND == 16) {
      u32x4 v[8];
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("ds_read_b128 %0, %1" : "=v"(v[s]) : "v"(off[s]));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("" :: "v"(v[s]));
      if (it == iters - 1) keep = v[0][0];
    } else if (KIND == 4) {
      uint32_t v[8];
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("ds_read_b32 %0, %1" : "=v"(v[s]) : "v"(off[s]));
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("" :: "v"(v[s]));
      if (it == iters - 1) keep = v[0];
    } else {
      u32x2 v[8];
#pragma unroll
      for (int s = 0; s < 8; s++) {
        if (KIND == -8) asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v[s]) : "v"(off[s]));
        else asm volatile("ds_read_b64 %0, %1" : "=v"(v[s]) : "v"(off[s]));
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int s = 0; s < 8; s++) asm volatile("" :: "v"(v[s]));
      if (it == iters - 1) keep = v[0][0];
    }
  }
  const int64_t c1 = (int64_t)clock64(), t1 = (int64_t)wall_clock64();
  if (threadIdx.x == 0) { out[2 * blockIdx.x] = c1 - c0; out[2 * blockIdx.x + 1] = t1 - t0; }
  if (keep == 0x12345678u && tile[threadIdx.x] == 77u) out[0] = 0;
}

}  // namespace

// iters rounds of 16 MFMAs per wave; grid workgroups of `waves` wavefronts (4 = one per SIMD, 8 = two per SIMD)
FDLC_API int fdlc_mfma_bf16(int grid, int waves, int iters, float* out, void* stream) {
  if (grid < 1 || iters < 1 || (waves != 4 && waves != 8) || out == nullptr) return 1;
  if (waves == 4) hipLaunchKernelGGL((mfma_bf16_kernel<4, 4>), dim3(grid), dim3(256), 0, (hipStream_t)stream, iters, out);
  else hipLaunchKernelGGL((mfma_bf16_kernel<2, 8>), dim3(grid), dim3(512), 0, (hipStream_t)stream, iters, out);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
FDLC_API double fdlc_mfma_bf16_flop(int grid, int waves, int iters) {
  return (double)grid * waves * iters * (waves == 4 ? 16.0 : 8.0) * (2.0 * 32 * 32 * 16);
}
// iters rounds of 16 v_mfma_f64_16x16x4_f64 per wave, grid workgroups of four wavefronts
FDLC_API int fdlc_mfma_f64(int grid, int iters, float* out, void* stream) {
  if (grid < 1 || iters < 1 || out == nullptr) return 1;
  hipLaunchKernelGGL(mfma_f64_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, iters, out);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
FDLC_API double fdlc_mfma_f64_flop(int grid, int iters) { return (double)grid * 4 * iters * 16.0 * (2.0 * 16 * 16 * 4); }
FDLC_API int fdlc_stream_read(const void* src, int64_t bytes, int grid, void* sink, void* stream) {
  if (!src || !sink || bytes < 16 || bytes % 16 || grid < 1) return 1;
  hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(kStreamThreads), 0, (hipStream_t)stream, (const u32x4*)src, bytes / 16, (uint32_t*)sink);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
FDLC_API int fdlc_stream_write(void* dst, int64_t bytes, int grid, void* stream) {
  if (!dst || bytes < 16 || bytes % 16 || grid < 1) return 1;
  hipLaunchKernelGGL(stream_write_kernel, dim3(grid), dim3(kStreamThreads), 0, (hipStream_t)stream, (u32x4*)dst, bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
FDLC_API int fdlc_stream_copy(void* dst, const void* src, int64_t bytes, int grid, void* stream) {
  if (!dst || !src || bytes < 16 || bytes % 16 || grid < 1) return 1;
  hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(kStreamThreads), 0, (hipStream_t)stream, (u32x4*)dst, (const u32x4*)src, bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
FDLC_API int fdlc_stream_mix21(void* dst, const void* a, const void* b, int64_t bytes, int grid, void* stream) {
  if (!dst || !a || !b || bytes < 16 || bytes % 16 || grid < 1) return 1;
  hipLaunchKernelGGL(stream_mix21_kernel, dim3(grid), dim3(kStreamThreads), 0, (hipStream_t)stream, (u32x4*)dst, (const u32x4*)a,
                     (const u32x4*)b, bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
// out: 2 * grid int64 (device).  Bytes one instruction of the pattern moves per wavefront: see fdlc_lds_probe_bytes.
FDLC_API int fdlc_lds_probe(int pattern, int grid, int iters, int64_t* out, void* stream) {
  if (pattern < 0 || pattern >= LDS_PATTERNS || grid < 1 || iters < 1 || out == nullptr) return 1;
  hipStream_t s = (hipStream_t)stream;
  switch (pattern) {
    case 0: hipLaunchKernelGGL(lds_probe_kernel<0>, dim3(grid), dim3(256), 0, s, iters, out); break;
    case 1: hipLaunchKernelGGL(lds_probe_kernel<1>, dim3(grid), dim3(256), 0, s, iters, out); break;
    case 2: hipLaunchKernelGGL(lds_probe_kernel<2>, dim3(grid), dim3(256), 0, s, iters, out); break;
    case 3: hipLaunchKernelGGL(lds_probe_kernel<3>, dim3(grid), dim3(256), 0, s, iters, out); break;
    case 4: hipLaunchKernelGGL(lds_probe_kernel<4>, dim3(grid), dim3(256), 0, s, iters, out); break;
    case 5: hipLaunchKernelGGL(lds_probe_kernel<5>, dim3(grid), dim3(256), 0, s, iters, out); break;
    case 6: hipLaunchKernelGGL(lds_probe_kernel<6>, dim3(grid), dim3(256), 0, s, iters, out); break;
    case 7: hipLaunchKernelGGL(lds_probe_kernel<7>, dim3(grid), dim3(256), 0, s, iters, out); break;
    case 8: hipLaunchKernelGGL(lds_probe_kernel<8>, dim3(grid), dim3(256), 0, s, iters, out); break;
    default: hipLaunchKernelGGL(lds_probe_kernel<9>, dim3(grid), dim3(256), 0, s, iters, out); break;
  }
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
// offsets: device array [8][64] of byte offsets; kind: 16, 8, 4 or -8 (see lds_probe_table_kernel)
FDLC_API int fdlc_lds_probe_table(const uint32_t* offsets, int kind, int grid, int iters, int64_t* out, void* stream) {
  if (offsets == nullptr || grid < 1 || iters < 1 || out == nullptr) return 1;
  hipStream_t s = (hipStream_t)stream;
  switch (kind) {
    case 16: hipLaunchKernelGGL(lds_probe_table_kernel<16>, dim3(grid), dim3(256), 0, s, offsets, iters, out); break;
    case 8: hipLaunchKernelGGL(lds_probe_table_kernel<8>, dim3(grid), dim3(256), 0, s, offsets, iters, out); break;
    case 4: hipLaunchKernelGGL(lds_probe_table_kernel<4>, dim3(grid), dim3(256), 0, s, offsets, iters, out); break;
    case -8: hipLaunchKernelGGL(lds_probe_table_kernel<-8>, dim3(grid), dim3(256), 0, s, offsets, iters, out); break;
    default: return 1;
  }
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
FDLC_API int fdlc_lds_probe_bytes(int pattern) {
  switch (pattern) {
    case 3: case 5: case 9: return 64 * 8;
    case 6: return 64 * 4;
    default: return 64 * 16;
  }
}
FDLC_API const char* fdlc_lds_probe_name(int pattern) {
  static const char* names[] = {"ds_read_b128 linear (lane*16)", "ds_read_b128 GEMM fragment, 128-byte rows (BK=64 swizzle)",
                                "ds_read_b128 GEMM fragment, 64-byte rows (BK=32 swizzle)", "ds_read_b64_tr_b16 GEMM fragment (r-major tile)",
                                "ds_read_b128 all lanes on the same banks (stride 512)", "ds_read_b64 linear (lane*8)",
                                "ds_read_b32 linear (lane*4)", "ds_read_b128 128-byte rows, former 32-bank swizzle",
                                "ds_read_b128 64-byte rows, former 32-bank swizzle", "ds_read_b64_tr_b16 r-major tile, former 32-bank swizzle"};
  return (pattern >= 0 && pattern < LDS_PATTERNS) ? names[pattern] : "?";
}
