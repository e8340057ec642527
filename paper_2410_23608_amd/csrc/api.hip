// Error reporting, version, the launch options and the one workspace query of libspa.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "spa_common.h"

namespace spa {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SPA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return SPA_OK;
}

// ---- launch options -------------------------------------------------------------------
// Parsed once: when the library is loaded (from the environment variable SPA_<NAME IN CAPITALS>
// of each option) and whenever spa_set_option is called.  The launch code reads the parsed
// integers only; nothing on the launch path touches the environment or a string.
static bool parse_option(Options& o, const char* name, const char* value) {
  const char* v = value != nullptr ? value : "";
  if (!std::strcmp(name, "attn_fwd_short")) {          // "" | words of: whole, 64, plain
    o.fwd_whole = std::strstr(v, "whole") != nullptr;
    o.fwd_step64 = std::strstr(v, "64") != nullptr;
    o.fwd_plain = std::strstr(v, "plain") != nullptr;
  } else if (!std::strcmp(name, "attn_fwd_long")) {    // "" (one query chain per wave) | "two"
    o.fwd_long_two = v[0] == 't';
  } else if (!std::strcmp(name, "attn_fwd_cfg")) {     // "" | "NW,BN" with NW in {2,4}, BN in {64,128}
    int a = 0, b = 0;
    o.fwd_nw = o.fwd_bn = 0;
    if (v[0] != 0) {
      if (std::sscanf(v, "%d,%d", &a, &b) != 2 || !(a == 2 || a == 4) || !(b == 64 || b == 128)) return false;
      o.fwd_nw = a;
      o.fwd_bn = b;
    }
  } else if (!std::strcmp(name, "attn_fwd_wave_max")) { // longest segment the one-wave kernels take
    const int n = v[0] != 0 ? std::atoi(v) : 256;
    if (n < 0 || n > 256) return false;
    o.fwd_wave_max = n;
  } else if (!std::strcmp(name, "attn_bwd_short")) {   // "" | "split" | "tiled"
    o.bwd_short = v[0] == 's' ? 1 : v[0] == 't' ? 2 : 0;
  } else if (!std::strcmp(name, "attn_bwd_long")) {    // "" | "two"
    o.bwd_long_two = v[0] == 't';
  } else if (!std::strcmp(name, "gemm_tm")) {          // 0 | 2 | 4 | 8
    const int n = std::atoi(v);
    if (!(n == 0 || n == 2 || n == 4 || n == 8)) return false;
    o.gemm_tm = n;
  } else if (!std::strcmp(name, "gemm_splits")) {      // 0 (automatic) .. 16
    const int n = std::atoi(v);
    if (n < 0 || n > 16) return false;
    o.gemm_splits = n;
  } else if (!std::strcmp(name, "pack_tile")) {        // 0 (automatic) | 16 .. 256
    const int n = std::atoi(v);
    if (!(n == 0 || n == 16 || n == 32 || n == 64 || n == 128 || n == 256)) return false;
    o.pack_tile = n;
  } else {
    return false;
  }
  return true;
}

static const char* const kOptionNames[] = {"attn_fwd_short", "attn_fwd_long", "attn_fwd_cfg", "attn_fwd_wave_max", "attn_bwd_short",
                                           "attn_bwd_long",  "gemm_tm",      "gemm_splits",       "pack_tile"};

static Options load_options() {
  Options o = {};
  o.fwd_wave_max = 256;
  for (const char* name : kOptionNames) {
    char env[64] = "SPA_";
    size_t n = std::strlen(env);
    for (const char* c = name; *c != 0 && n + 1 < sizeof(env); ++c) env[n++] = (char)(*c >= 'a' && *c <= 'z' ? *c - 32 : *c);
    env[n] = 0;
    if (const char* v = std::getenv(env)) {
      Options trial = o;
      if (parse_option(trial, name, v)) o = trial;     // a malformed variable is ignored
    }
  }
  return o;
}

static Options g_options = load_options();

const Options& options() { return g_options; }

}  // namespace spa

extern "C" int spa_version(void) { return 200; }

extern "C" const char* spa_last_error(void) { return spa::g_err; }

extern "C" int spa_set_option(const char* name, const char* value) {
  SPA_REQUIRE(name != nullptr, SPA_ERR_INVALID_ARG, "spa_set_option: name is null");
  spa::Options trial = spa::g_options;
  SPA_REQUIRE(spa::parse_option(trial, name, value), SPA_ERR_INVALID_ARG,
              "spa_set_option: unknown option or bad value: %s = \"%s\"", name, value != nullptr ? value : "");
  spa::g_options = trial;
  return SPA_OK;
}

extern "C" size_t spa_workspace_bytes(int op, int B, int N, int C, int H, int dtype) {
  if (B < 1 || N < 1 || C < 1 || H < 1 || C % H != 0) return 0;
  const long cap = (long)B * N;
  switch (op) {
    case SPA_OP_PACKED_ATTENTION_BWD: return spa_attention_bwd_workspace_bytes(B, N, H, C / H, dtype);
    case SPA_OP_GATE_BWD: return spa_gate_bwd_workspace_bytes(B, N, C, dtype);
    case SPA_OP_QKV_PROJECTION_BWD_WEIGHT:
      return cap < 2147483647L ? spa_linear_bwd_weight_workspace_bytes((int)cap, C, 3 * C, dtype) : 0;
    case SPA_OP_OUT_PROJECTION_BWD_WEIGHT:
      return cap < 2147483647L ? spa_linear_bwd_weight_workspace_bytes((int)cap, C, C, dtype) : 0;
    default: return 0;   // the forward calls and the row-moving transposes need none
  }
}
