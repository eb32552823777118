// Kernel-selection overrides.  The library that ships (built without FL_TEST_EXPORTS) has none:
// every launcher picks its kernel from the problem alone and the getters below are constants.
// The test build keeps one process-wide override per kernel family, so that a parity test can put a
// given problem on each tile variant, on the general attention kernels and on the two-kernel
// attention backward.
#include "kernels.h"

namespace fl {
#ifdef FL_TEST_EXPORTS
namespace {
int g_pipe_variant = -1;       // pipelined bf16 GEMM: -1 automatic, >= 0 that variant, -2 never
int g_tile_height = 0;         // register-staged GEMM: 0 automatic, 1 = 64x128 tiles, 2 = 128x128
bool g_general_attention = false;
bool g_unfused_attention_bwd = false;
}  // namespace
int forced_gemm_pipe_variant() { return g_pipe_variant; }
int forced_gemm_tile_height() { return g_tile_height; }
bool forced_general_attention() { return g_general_attention; }
bool forced_unfused_attention_bwd() { return g_unfused_attention_bwd; }
void gemm_pipe_force_variant(int v) { g_pipe_variant = v; }
void gemm_force_tile_height(int tmw) { g_tile_height = tmw; }
void attention_force_general(bool on) { g_general_attention = on; }
void attention_force_unfused_bwd(bool on) { g_unfused_attention_bwd = on; }
#else
int forced_gemm_pipe_variant() { return -1; }
int forced_gemm_tile_height() { return 0; }
bool forced_general_attention() { return false; }
bool forced_unfused_attention_bwd() { return false; }
#endif
}  // namespace fl
