// placeholder until the backward kernels land
#include "spa_common.h"
using namespace spa;
extern "C" size_t spa_attention_bwd_workspace_bytes(int, int, int, int, int) { return 0; }
extern "C" int spa_packed_attention_bwd(const void*, const void*, const void*, int64_t, const void*, const void*,
                                        const float*, const int32_t*, int, int, int, int, int, float, void*, void*,
                                        void*, int64_t, void*, size_t, void*) {
  return fail(SPA_ERR_UNSUPPORTED, "spa_packed_attention_bwd: not built yet");
}
extern "C" size_t spa_gate_bwd_workspace_bytes(int, int, int, int) { return 0; }
extern "C" int spa_gate_bwd(const void*, const void*, float, const float*, const float*, const uint8_t*, const void*,
                            int, float, int, int, int, int, float*, void*, float*, float*, void*, size_t, void*) {
  return fail(SPA_ERR_UNSUPPORTED, "spa_gate_bwd: not built yet");
}
