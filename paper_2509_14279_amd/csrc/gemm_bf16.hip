// bf16 fast path (placeholder: not enabled yet; every shape takes the generic kernels).
#include "common.hip.h"
#include "internal.h"

namespace fdl {
bool fast_f1_supported(int64_t, int64_t, int64_t) { return false; }
bool fast_b3_supported(int64_t, int64_t, int64_t) { return false; }
bool fast_b4_supported(int64_t, int64_t, int64_t) { return false; }
int fast_f1_stat_tile_w() { return 128; }
void launch_fast_f1(int64_t, int64_t, int64_t, const void*, const void*, const float*, void*, void*, hipStream_t) {}
void launch_transpose_bf16(int64_t, int64_t, const void*, void*, hipStream_t) {}
void launch_fast_b3(int64_t, int64_t, int64_t, const void*, const void*, void*, hipStream_t) {}
int fast_b4_split(int64_t, int64_t, int64_t) { return 1; }
void launch_fast_b4(int64_t, int64_t, int64_t, int, const void*, const void*, void*, void*, hipStream_t) {}
}  // namespace fdl
