// Host-side exercise of libspa under AddressSanitizer / UndefinedBehaviorSanitizer (no GPU needed):
// option parsing, workspace queries and the argument validation of the entry points, each of which
// must refuse bad arguments before it touches the HIP runtime.  Built and run by
// tests/test_host_sanitizers.py against the host-sanitized build of the library.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>

#include "spa.h"

static int failures = 0;
#define EXPECT(cond)                                                       \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);       \
      ++failures;                                                          \
    }                                                                      \
  } while (0)

// a refused call: negative code and a message that names the call
static void refused(int rc, const char* fn) {
  EXPECT(rc < 0);
  EXPECT(std::strstr(spa_last_error(), fn) != nullptr);
}

int main() {
  EXPECT(spa_version() >= 200);

  // ---- options: every name, good and bad values, long and empty strings
  const char* names[] = {"attn_fwd_short", "attn_fwd_long", "attn_fwd_cfg", "attn_fwd_wave_max", "attn_bwd_short",
                         "attn_bwd_long",  "gemm_tm",       "gemm_splits",  "pack_tile"};
  for (const char* n : names) {
    EXPECT(spa_set_option(n, nullptr) == SPA_OK);
    EXPECT(spa_set_option(n, "") == SPA_OK);
  }
  EXPECT(spa_set_option("attn_fwd_short", "whole 64 plain") == SPA_OK);
  EXPECT(spa_set_option("attn_fwd_cfg", "2,64") == SPA_OK);
  EXPECT(spa_set_option("attn_fwd_cfg", "3,64") == SPA_ERR_INVALID_ARG);
  EXPECT(spa_set_option("attn_fwd_cfg", "4") == SPA_ERR_INVALID_ARG);
  EXPECT(spa_set_option("attn_fwd_wave_max", "300") == SPA_ERR_INVALID_ARG);
  EXPECT(spa_set_option("gemm_tm", "3") == SPA_ERR_INVALID_ARG);
  EXPECT(spa_set_option("gemm_splits", "17") == SPA_ERR_INVALID_ARG);
  EXPECT(spa_set_option("pack_tile", "48") == SPA_ERR_INVALID_ARG);
  EXPECT(spa_set_option("no_such_option", "1") == SPA_ERR_INVALID_ARG);
  EXPECT(spa_set_option(nullptr, "1") == SPA_ERR_INVALID_ARG);
  const std::string longv(5000, 'x');                      // the error message must be cut, not overrun
  EXPECT(spa_set_option(longv.c_str(), longv.c_str()) == SPA_ERR_INVALID_ARG);
  EXPECT(std::strlen(spa_last_error()) > 0);
  for (const char* n : names) EXPECT(spa_set_option(n, nullptr) == SPA_OK);

  // ---- workspace queries: every op, sizes from tiny to large, bad arguments give 0
  for (int op = -1; op <= 9; ++op)
    for (int dtype = -1; dtype <= 2; ++dtype) {
      (void)spa_workspace_bytes(op, 64, 196, 768, 12, dtype);
      (void)spa_workspace_bytes(op, 16, 3136, 96, 3, dtype);
      EXPECT(spa_workspace_bytes(op, 0, 196, 768, 12, dtype) == 0);
      EXPECT(spa_workspace_bytes(op, 64, -5, 768, 12, dtype) == 0);
    }
  EXPECT(spa_workspace_bytes(SPA_OP_GATE_BWD, 64, 196, 768, 12, SPA_BF16) == spa_gate_bwd_workspace_bytes(64, 196, 768, SPA_BF16));
  EXPECT(spa_workspace_bytes(SPA_OP_PACKED_ATTENTION_BWD, 16, 3136, 96, 3, SPA_BF16) ==
         spa_attention_bwd_workspace_bytes(16, 3136, 3, 32, SPA_BF16));
  EXPECT(spa_workspace_bytes(SPA_OP_GATE_SELECT, 64, 196, 768, 12, SPA_BF16) == 0);
  EXPECT(spa_attention_bwd_workspace_bytes(2147483647, 2147483647, 1, 64, SPA_BF16) > 0);   // no signed overflow
  (void)spa_linear_bwd_weight_workspace_bytes(2147483647, 768, 2304, SPA_BF16);
  (void)spa_gate_bwd_workspace_bytes(2147483647, 2147483647, 1024, SPA_F32);

  // ---- argument validation: nothing below may reach a kernel launch
  alignas(16) static unsigned char buf[4096];
  void* p = buf;
  float* f = reinterpret_cast<float*>(buf);
  int32_t* i32 = reinterpret_cast<int32_t*>(buf);
  uint8_t* u8 = buf;
  refused(spa_gate_select(nullptr, p, 0.f, nullptr, 0.5f, 2, 196, 64, SPA_F32, f, u8, nullptr, nullptr), "spa_gate_select");
  refused(spa_gate_select(p, p, 0.f, nullptr, 1.5f, 2, 196, 64, SPA_F32, f, u8, nullptr, nullptr), "spa_gate_select");
  refused(spa_gate_select(p, p, 0.f, nullptr, 0.5f, 2, 196, 64, 7, f, u8, nullptr, nullptr), "spa_gate_select");
  refused(spa_gate_select(p, p, 0.f, nullptr, 0.5f, -2, 196, 64, SPA_F32, f, u8, nullptr, nullptr), "spa_gate_select");
  refused(spa_gate_select_index(p, p, 0.f, nullptr, 0.5f, 2, 196, 64, SPA_F32, f, u8, nullptr, i32, i32, i32, nullptr, p, 16,
                                nullptr), "spa_gate_select_index");
  refused(spa_pack(p, nullptr, nullptr, nullptr, 2, 196, 64, SPA_F32, 0, p, i32, i32, i32, i32, nullptr), "spa_pack");
  refused(spa_pack(p, u8, nullptr, nullptr, 2, 196, 63, SPA_BF16, 0, p, i32, i32, i32, i32, nullptr), "spa_pack");
  refused(spa_packed_attention(p, p, p, 64, 64, 64, i32, 2, 196, 2, 48, SPA_BF16, 0.f, p, nullptr, nullptr), "spa_packed_attention");
  refused(spa_packed_attention(p, p, p, 60, 64, 64, i32, 2, 196, 2, 32, SPA_BF16, 0.f, p, nullptr, nullptr), "spa_packed_attention");
  refused(spa_packed_attention(buf + 2, p, p, 64, 64, 64, i32, 2, 196, 2, 32, SPA_BF16, 0.f, p, nullptr, nullptr),
          "spa_packed_attention");
  refused(spa_packed_attention(p, p, p, 64, 64, 64, nullptr, 2, 196, 2, 32, SPA_BF16, 0.f, p, nullptr, nullptr), "spa_packed_attention");
  refused(spa_packed_attention(p, p, p, 64, 64, (int64_t)1 << 40, i32, 2, 196, 2, 32, SPA_BF16, 0.f, p, nullptr, nullptr),
          "spa_packed_attention");
  refused(spa_packed_attention(p, p, p, 64, 64, 64, i32, 2, 196, 2, 32, SPA_BF16, -1.f, p, nullptr, nullptr), "spa_packed_attention");
  refused(spa_selected_attention_unpack(p, p, p, 64, 64, 64, u8, nullptr, 2, 300, 2, 32, SPA_BF16, 0.f, p, nullptr),
          "spa_selected_attention_unpack");
  refused(spa_selected_attention_unpack(p, p, p, 96, 96, 96, u8, nullptr, 2, 196, 2, 48, SPA_F32, 0.f, p, nullptr),
          "spa_selected_attention_unpack");
  refused(spa_selected_attention_unpack(p, p, p, 64, 64, 64, nullptr, nullptr, 2, 196, 2, 32, SPA_BF16, 0.f, p, nullptr),
          "spa_selected_attention_unpack");
  refused(spa_unpack(nullptr, i32, nullptr, 2, 196, 64, SPA_F32, p, nullptr), "spa_unpack");
  refused(spa_maxpool2x2(f, 2, 7, 7, f, nullptr), "spa_maxpool2x2");
  refused(spa_packed_attention_bwd(p, p, p, 64, 64, 64, p, p, f, i32, 2, 300, 2, 32, SPA_BF16, 0.f, p, p, p, 64, 64, 64, nullptr, 0,
                                   nullptr), "spa_packed_attention_bwd");
  refused(spa_gate_bwd(p, p, 0.f, f, nullptr, u8, nullptr, 0, 1.f, 2, 196, 64, SPA_F32, f, p, f, f, nullptr, 0, nullptr), "spa_gate_bwd");
  refused(spa_gate_bwd_static(p, p, 0.f, f, nullptr, u8, nullptr, 0, 1.f, 2, 196, 4096, SPA_F32, f, p, f, f, nullptr),
          "spa_gate_bwd_static");
  refused(spa_ceiling_copy(nullptr, p, 1024, nullptr), "spa_ceiling_copy");

  std::printf(failures == 0 ? "host sanitizer driver: ok\n" : "host sanitizer driver: %d failure(s)\n", failures);
  return failures == 0 ? 0 : 1;
}
