"""The C-ABI library loads and exports every symbol include/spa.h declares; argument
validation answers before anything is launched (so it can be exercised without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2410_23608_amd", "libspa.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2410_23608_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "spa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spa_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"spa_gate_select", "spa_pack", "spa_packed_attention", "spa_unpack"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in spa.h but not exported"


def test_binding_covers_every_declared_symbol(lib):
    src = open(os.path.join(ROOT, "paper_2410_23608_amd", "spa.py")).read()
    for n in declared_functions():
        assert f'"{n}"' in src, f"binding lacks {n}"


def test_version_and_validation_without_gpu(lib):
    lib.spa_version.restype = ctypes.c_int
    assert lib.spa_version() >= 100
    lib.spa_last_error.restype = ctypes.c_char_p
    P = ctypes.c_void_p
    lib.spa_gate_select.restype = ctypes.c_int
    lib.spa_gate_select.argtypes = [P, P, ctypes.c_float, P, ctypes.c_float] + [ctypes.c_int] * 4 + [P] * 4
    assert lib.spa_gate_select(None, None, 0.0, None, 0.5, 1, 1, 8, 0, None, None, None, None) == -1
    assert b"null" in lib.spa_last_error()
    # a non-null but never dereferenced pointer: the tau check fires before any launch
    fake = ctypes.c_void_p(4096)
    assert lib.spa_gate_select(fake, fake, 0.0, None, 1.0, 1, 1, 8, 0, fake, fake, None, None) == -1
    assert b"tau" in lib.spa_last_error()
    assert lib.spa_gate_select(fake, fake, 0.0, None, 0.5, 1, 1, 7, 0, fake, fake, None, None) == -1
    assert b"multiple of 16" in lib.spa_last_error()
    assert lib.spa_gate_select(fake, fake, 0.0, None, 0.5, 1, 1, 8, 5, fake, fake, None, None) == -2
    lib.spa_packed_attention.restype = ctypes.c_int
    lib.spa_packed_attention.argtypes = [P, P, P, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, P] + [ctypes.c_int] * 5 + [ctypes.c_float, P, P, P]
    assert lib.spa_packed_attention(fake, fake, fake, 48, 48, 48, fake, 1, 8, 2, 24, 1, 0.0, fake, None, None) == -2
    assert b"head dim" in lib.spa_last_error()


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2410_23608_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b|oracle/|spa_oracle", text, flags=re.M), f


def test_validation_of_the_wider_entry_points_without_gpu(lib):
    """Argument checks of the entry points beyond the four hot-path calls answer before any
    launch (no GPU needed): bad grids, capacities, temperatures, missing index arrays."""
    lib.spa_last_error.restype = ctypes.c_char_p
    P, I, F, L = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_int64
    fake = ctypes.c_void_p(4096)

    lib.spa_pack_shifted.restype = I
    lib.spa_pack_shifted.argtypes = [P, P, P, P] + [I] * 8 + [P] * 6
    assert lib.spa_pack_shifted(None, fake, None, None, 1, 0, 4, 1, 1, 8, 1, 0, None, fake, fake, fake, fake, None) == -1
    assert b"grid_h" in lib.spa_last_error()

    lib.spa_container_segments_capacity.restype = L
    lib.spa_container_segments_capacity.argtypes = [I, L, I]
    assert lib.spa_container_segments_capacity(64, 12544, 49) == 64 + 12544 // 49
    assert lib.spa_container_segments_capacity(0, 10, 4) == -1
    lib.spa_container_segments.restype = I
    lib.spa_container_segments.argtypes = [P, I, I, L, I, P, P, P]
    assert lib.spa_container_segments(fake, 4, 7, 100, 4 + 100 // 7 - 1, fake, fake, None) == -3     # one short
    assert b"seg_cap" in lib.spa_last_error()
    assert lib.spa_container_segments(fake, 4, 0, 100, 64, fake, fake, None) == -1

    lib.spa_gate_select_gumbel.restype = I
    lib.spa_gate_select_gumbel.argtypes = [P, P, F, P, P, F, F] + [I] * 4 + [P] * 4
    assert lib.spa_gate_select_gumbel(fake, fake, 0.0, None, None, 1.0, 0.5, 1, 1, 8, 0, fake, fake, None, None) == -1
    assert b"noise" in lib.spa_last_error()
    assert lib.spa_gate_select_gumbel(fake, fake, 0.0, None, fake, -1.0, 0.5, 1, 1, 8, 0, fake, fake, None, None) == -1
    assert b"temperature" in lib.spa_last_error()

    lib.spa_gate_select_pooled.restype = I
    lib.spa_gate_select_pooled.argtypes = [P, P, F, P, F] + [I] * 5 + [P] * 5
    assert lib.spa_gate_select_pooled(fake, fake, 0.0, None, 0.5, 1, 2, 2, 8, 0, fake, fake, None, None, None) == -1
    assert b"s_fine" in lib.spa_last_error()

    lib.spa_linear_packed.restype = I
    lib.spa_linear_packed.argtypes = [P] * 6 + [I] * 4 + [P, L, P]
    assert lib.spa_linear_packed(fake, None, fake, None, fake, None, 8, 64, 64, 1, fake, 64, None) == -1
    assert b"gather_idx" in lib.spa_last_error()
    assert lib.spa_linear_packed(fake, None, None, None, fake, None, 8, 60, 64, 1, fake, 64, None) == -2
    assert b"multiple of 8" in lib.spa_last_error()
    lib.spa_linear_packed_scatter.restype = I
    lib.spa_linear_packed_scatter.argtypes = [P] * 4 + [I] * 4 + [P, P, P, L, P]
    assert lib.spa_linear_packed_scatter(fake, None, fake, None, 8, 64, 64, 1, None, None, fake, 64, None) == -1
    assert b"scatter_idx" in lib.spa_last_error()

    lib.spa_packed_attention_bwd_tokens.restype = I
    lib.spa_packed_attention_bwd_tokens.argtypes = ([P, P, P, L, L, L, P, P, P, P] + [I] * 5 +
                                                    [F, P, P, L, P, P, P, L, L, L, P, ctypes.c_size_t, P])
    tok_args = lambda dtype, n_max, gidx: (fake, fake, fake, 64, 64, 64, fake, fake, fake, fake, 2, n_max, 1, 64, dtype,
                                           0.0, gidx, fake, 2 * n_max, fake, fake, fake, 64, 64, 64, None, 0, None)
    assert lib.spa_packed_attention_bwd_tokens(*tok_args(1, 64, None)) == -1
    assert lib.spa_packed_attention_bwd_tokens(*tok_args(0, 64, fake)) == -3          # fp32 needs the workspace
    assert lib.spa_packed_attention_bwd_tokens(*tok_args(1, 257, fake)) == -3         # long segments need the workspace
    assert b"workspace" in lib.spa_last_error()

    lib.spa_linear_packed_bwd_input.restype = I
    lib.spa_linear_packed_bwd_input.argtypes = [P, P, L, P, P, I, I, I, I, P, P, L, P, L, P]
    assert lib.spa_linear_packed_bwd_input(fake, None, 64, None, fake, 8, 64, 64, 1, None, fake, 8, fake, 64, None) == -1
    assert b"dx_idx" in lib.spa_last_error()
    assert lib.spa_linear_packed_bwd_input(fake, None, 64, None, fake, 8, 60, 64, 1, None, None, 0, fake, 64, None) == -2
    lib.spa_linear_bwd_weight_workspace_bytes.restype = ctypes.c_size_t
    lib.spa_linear_bwd_weight_workspace_bytes.argtypes = [I] * 4
    need = lib.spa_linear_bwd_weight_workspace_bytes(12544, 384, 1152, 1)
    assert need >= (384 * 1152 + 1152) * 4 and need % 256 == 0
    assert lib.spa_linear_bwd_weight_workspace_bytes(12544, 384, 1152, 0) == 0          # fp32 needs none
    lib.spa_linear_packed_bwd_weight.restype = I
    lib.spa_linear_packed_bwd_weight.argtypes = [P, P, L, P, P, P, P, I, I, I, I, P, P, P, ctypes.c_size_t, P]
    assert lib.spa_linear_packed_bwd_weight(fake, None, 64, fake, None, None, None, 8, 64, 64, 1, fake, None, None, 0, None) == -3
    assert b"workspace" in lib.spa_last_error()
    assert lib.spa_linear_packed_bwd_weight(fake, None, 64, fake, None, fake, None, 8, 64, 64, 1, fake, None, None, 0, None) == -1
    assert b"x_idx" in lib.spa_last_error()

    lib.spa_pack_pair.restype = I
    lib.spa_pack_pair.argtypes = [P, I, P, I, P, P, P, I, I, I, P, P, P, P, P, P, P]
    assert lib.spa_pack_pair(fake, 64, None, 64, fake, None, None, 1, 8, 1, fake, fake, None, None, None, None, None) == -1
    assert b"null" in lib.spa_last_error()
    assert lib.spa_pack_pair(fake, 64, fake, 12, fake, None, None, 1, 8, 1, fake, fake, None, None, None, None, None) == -1
    assert b"multiple of 16" in lib.spa_last_error()

    lib.spa_ceiling_mfma.restype = ctypes.c_double
    lib.spa_ceiling_mfma.argtypes = [P, I, I, P]
    assert lib.spa_ceiling_mfma(None, 1, 1, None) == -1.0


def test_options_and_the_single_workspace_query_without_gpu(lib):
    """spa_set_option parses once and rejects unknown names / malformed values; spa_workspace_bytes
    agrees with the per-call queries."""
    I = ctypes.c_int
    lib.spa_last_error.restype = ctypes.c_char_p
    lib.spa_set_option.restype = I
    lib.spa_set_option.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    assert lib.spa_set_option(b"attn_fwd_short", b"whole") == 0
    assert lib.spa_set_option(b"attn_fwd_short", None) == 0
    assert lib.spa_set_option(b"attn_fwd_cfg", b"4,128") == 0 and lib.spa_set_option(b"attn_fwd_cfg", b"") == 0
    assert lib.spa_set_option(b"attn_fwd_cfg", b"3,128") == -1 and b"attn_fwd_cfg" in lib.spa_last_error()
    assert lib.spa_set_option(b"no_such_option", b"1") == -1
    assert lib.spa_set_option(b"pack_tile", b"48") == -1 and lib.spa_set_option(b"pack_tile", b"0") == 0
    assert lib.spa_set_option(None, b"1") == -1
    S = ctypes.c_size_t
    lib.spa_workspace_bytes.restype = S
    lib.spa_workspace_bytes.argtypes = [I] * 6
    for f, n in (("spa_attention_bwd_workspace_bytes", 5), ("spa_gate_bwd_workspace_bytes", 4),
                 ("spa_linear_bwd_weight_workspace_bytes", 4)):
        getattr(lib, f).restype = S
        getattr(lib, f).argtypes = [I] * n
    B, N, C, H = 64, 196, 768, 12
    assert lib.spa_workspace_bytes(4, B, N, C, H, 1) == lib.spa_attention_bwd_workspace_bytes(B, N, H, C // H, 1) > 0
    assert lib.spa_workspace_bytes(5, B, N, C, H, 1) == lib.spa_gate_bwd_workspace_bytes(B, N, C, 1) > 0
    assert lib.spa_workspace_bytes(6, B, N, C, H, 1) == lib.spa_linear_bwd_weight_workspace_bytes(B * N, C, 3 * C, 1) > 0
    assert lib.spa_workspace_bytes(7, B, N, C, H, 1) == lib.spa_linear_bwd_weight_workspace_bytes(B * N, C, C, 1) > 0
    for op in (0, 1, 2, 3, 99):
        assert lib.spa_workspace_bytes(op, B, N, C, H, 1) == 0
    assert lib.spa_workspace_bytes(4, 0, N, C, H, 1) == 0 and lib.spa_workspace_bytes(4, B, N, C, 5, 1) == 0
