"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
rejects bad arguments before touching the GPU.  No compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2505_11432_amd", "libmoe_hip.so")
HEADER = os.path.join(ROOT, "include", "moe.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2505_11432_amd.build import ensure_built
    ensure_built()
    return ctypes.CDLL(LIB)


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert {"moe_route", "moe_dispatch", "moe_expert_ffn_fwd", "moe_expert_ffn_bwd", "moe_combine",
            "moe_quant_fp8"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_covers_every_export(lib):
    from paper_2505_11432_amd import binding
    assert sorted(binding.EXPORTS) == declared_symbols()
    assert binding.moe_abi_version() == 1


def test_status_strings(lib):
    lib.moe_status_string.restype = ctypes.c_char_p
    assert lib.moe_status_string(0) == b"ok"
    for s in (-1, -2, -3, -4):
        assert len(lib.moe_status_string(s)) > 3


def test_workspace_bytes(lib):
    lib.moe_workspace_bytes.restype = ctypes.c_size_t
    assert lib.moe_workspace_bytes(256, 128, 8, 2, 256, 0) >= 512 * 4 * 256 * 4
    assert lib.moe_workspace_bytes(8192, 4096, 8, 2, 14336, 1) >= 16384 * 4 * 14336 * 2
    assert lib.moe_workspace_bytes(8, 128, 8, 9, 256, 1) == 0          # k > E
    assert lib.moe_workspace_bytes(8, 128, 300, 2, 256, 1) == 0        # E too large
    assert lib.moe_workspace_bytes(-1, 128, 8, 2, 256, 1) == 0


def test_argument_errors_without_gpu(lib):
    P = ctypes.c_void_p
    null = P(0)
    fake = P(4096)     # non-NULL, aligned; never dereferenced because validation fails first
    # route: k > E, NULL logits, missing workspace
    assert lib.moe_route(fake, 4, 8, 9, 1, fake, fake, fake, fake, fake, fake, fake, ctypes.c_size_t(1 << 20), null) == -1
    assert lib.moe_route(null, 4, 8, 2, 1, fake, fake, fake, fake, fake, fake, fake, ctypes.c_size_t(1 << 20), null) == -1
    assert lib.moe_route(fake, 4, 8, 2, 1, fake, fake, fake, fake, fake, fake, null, ctypes.c_size_t(0), null) == -3
    assert lib.moe_route(fake, 4, 8, 2, 1, fake, fake, fake, fake, fake, fake, fake, ctypes.c_size_t(8), null) == -3
    assert lib.moe_route(fake, 0, 8, 2, 1, null, null, null, null, null, null, null, ctypes.c_size_t(0), null) == 0
    # dispatch: d not a multiple of 16, bad dtype, misaligned pointer, fp8 without scales
    assert lib.moe_dispatch(fake, null, 1, fake, null, 4, 2, 24, fake, null, null) == -2
    assert lib.moe_dispatch(fake, null, 7, fake, null, 4, 2, 32, fake, null, null) == -2
    assert lib.moe_dispatch(P(4100), null, 1, fake, null, 4, 2, 32, fake, null, null) == -2
    assert lib.moe_dispatch(fake, null, 2, fake, null, 4, 2, 32, fake, null, null) == -1
    assert lib.moe_dispatch(null, null, 1, fake, null, 4, 2, 32, fake, null, null) == -1
    assert lib.moe_dispatch(null, null, 1, null, null, 0, 2, 32, null, null, null) == 0
    # combine: fp32 rows cannot be written as bf16; fp8 needs scales
    assert lib.moe_combine(fake, null, 0, fake, null, 4, 2, 32, fake, 1, null) == -2
    assert lib.moe_combine(fake, null, 2, fake, null, 4, 2, 32, fake, 1, null) == -1
    # expert ffn: E out of range, f misaligned, workspace too small
    Z = ctypes.c_size_t
    assert lib.moe_expert_ffn_fwd(fake, null, 1, fake, fake, null, fake, null, 1, 64, 32, 0, 32, fake, fake, null, 1, null, null, fake, Z(1 << 30), null) == -1
    assert lib.moe_expert_ffn_fwd(fake, null, 1, fake, fake, null, fake, null, 1, 64, 32, 4, 24, fake, fake, null, 1, null, null, fake, Z(1 << 30), null) == -2
    assert lib.moe_expert_ffn_fwd(fake, null, 1, fake, fake, null, fake, null, 1, 64, 32, 4, 32, fake, fake, null, 1, null, null, fake, Z(16), null) == -3
    assert lib.moe_expert_ffn_bwd(fake, fake, fake, null, fake, fake, fake, 1, 64, 32, 4, 32, fake, fake, fake, 0, 0, fake, Z(16), null) == -3
    assert lib.moe_expert_ffn_bwd(fake, fake, fake, null, fake, fake, fake, 0, 64, 32, 4, 32, fake, fake, fake, 1, 0, fake, Z(1 << 30), null) == -2
    # quant: bad mode, misaligned columns
    assert lib.moe_quant_fp8(fake, 1, 4, 32, 5, fake, fake, null) == -1
    assert lib.moe_quant_fp8(fake, 1, 4, 20, 0, fake, fake, null) == -2
    assert lib.moe_quant_fp8(null, 1, 0, 32, 0, null, null, null) == 0


def test_fp8_backward_argument_errors_without_gpu(lib):
    from paper_2505_11432_amd.binding import FfnBwdFp8Args
    P, L = ctypes.c_void_p, ctypes.c_long
    null, fake = P(0), P(4096)
    lib.moe_tgroup_tokens.restype = ctypes.c_size_t
    assert lib.moe_tgroup_tokens(16384, 8) == (128 + 8) * 128
    assert lib.moe_tgroup_tokens(130, 3) == (2 + 3) * 128
    assert lib.moe_tgroup_tokens(-1, 3) == 0
    # token-group cast: leading dimension too small / not a multiple of 128, columns not a multiple of 16, NULL offsets
    assert lib.moe_quant_fp8_tgroup(fake, 1, 256, 64, fake, 2, fake, fake, L(384), fake, null) == -1
    assert lib.moe_quant_fp8_tgroup(fake, 1, 256, 64, fake, 2, fake, fake, L(520), fake, null) == -1
    assert lib.moe_quant_fp8_tgroup(fake, 1, 256, 24, fake, 2, fake, fake, L(512), fake, null) == -2
    assert lib.moe_quant_fp8_tgroup(fake, 1, 256, 64, null, 2, fake, fake, L(512), fake, null) == -1
    lib.moe_expert_ffn_bwd_fp8.argtypes = [ctypes.POINTER(FfnBwdFp8Args), P]
    assert lib.moe_expert_ffn_bwd_fp8(None, null) == -1
    a = FfnBwdFp8Args()
    for name, _ in FfnBwdFp8Args._fields_:
        if name not in ("M", "d", "E", "f", "grad_dt", "accumulate", "ldt"):
            setattr(a, name, 4096)
    a.M, a.d, a.E, a.f, a.grad_dt, a.accumulate, a.ldt = 256, 64, 2, 32, 0, 0, 512
    a.ldt = 384                                       # too small for 256 rows and 2 experts
    assert lib.moe_expert_ffn_bwd_fp8(ctypes.byref(a), null) == -1
    a.ldt = 512
    a.f = 24
    assert lib.moe_expert_ffn_bwd_fp8(ctypes.byref(a), null) == -2
    a.f = 32
    a.dh_t = None
    assert lib.moe_expert_ffn_bwd_fp8(ctypes.byref(a), null) == -1
    a.dh_t = 4100                                     # misaligned
    assert lib.moe_expert_ffn_bwd_fp8(ctypes.byref(a), null) == -2


def test_route_range_capacity_balance_argument_errors_without_gpu(lib):
    P, Z, F = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
    null, fake = P(0), P(4096)
    big = Z(1 << 24)
    # expert range outside [0, E] or reversed
    assert lib.moe_route_range(fake, 4, 8, 2, 1, 3, 9, fake, fake, fake, fake, fake, fake, fake, big, null) == -1
    assert lib.moe_route_range(fake, 4, 8, 2, 1, 5, 4, fake, fake, fake, fake, fake, fake, fake, big, null) == -1
    assert lib.moe_route_range(fake, 4, 8, 2, 1, 2, 6, fake, fake, fake, fake, fake, fake, null, Z(0), null) == -3
    # devices must divide the experts; capacity >= 0; score is required; workspace size
    lib.moe_route_capacity_workspace_bytes.restype = Z
    need = lib.moe_route_capacity_workspace_bytes(64, 8, 2)
    assert need > 64 * 2 and lib.moe_route_capacity_workspace_bytes(64, 8, 9) == 0
    args = lambda g, cap, score, ws, n: (fake, 64, 8, 2, 1, g, cap, fake, fake, score, fake, fake, fake, fake, ws, Z(n), null)
    assert lib.moe_route_capacity(*args(3, 10, fake, fake, need)) == -1
    assert lib.moe_route_capacity(*args(4, -1, fake, fake, need)) == -1
    assert lib.moe_route_capacity(*args(4, 10, null, fake, need)) == -1
    assert lib.moe_route_capacity(*args(4, 10, fake, fake, need - 1)) == -3
    lib.moe_balance_loss.argtypes = [P, P, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, F, P, P, P, P, Z, P]
    assert lib.moe_balance_loss(fake, fake, 64, 8, 2, 3, F(0.1), fake, fake, fake, fake, big, null) == -1
    assert lib.moe_balance_loss(fake, fake, 64, 8, 2, 4, F(0.1), null, fake, fake, fake, big, null) == -1
    assert lib.moe_balance_loss(fake, fake, 64, 8, 2, 4, F(0.1), fake, fake, fake, null, Z(0), null) == -3
    lib.moe_balance_loss_bwd.argtypes = [P, P, ctypes.c_int, ctypes.c_int, ctypes.c_int, F, P, P]
    assert lib.moe_balance_loss_bwd(fake, fake, 64, 8, 5, F(0.1), fake, null) == -1
    assert lib.moe_balance_loss_bwd(fake, null, 64, 8, 4, F(0.1), fake, null) == -1
    assert lib.moe_balance_loss_bwd(null, null, 0, 8, 4, F(0.1), null, null) == 0


def test_fused_order_argument_errors_without_gpu(lib):
    P, Z, I = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    null, fake = P(0), P(4096)
    lib.moe_expert_ffn_fused_workspace_bytes.restype = Z
    need = lib.moe_expert_ffn_fused_workspace_bytes(64, 2, 128, 256)
    # A' + dH + one [M,d] buffer + gate-gradient partials + split-K scratch
    assert need >= 128 * 256 * 2 + 128 * 512 * 2 + 128 * 128 * 2 + 4 * 128 * 4 + 256 * 256 * 256 * 4
    assert lib.moe_expert_ffn_fused_workspace_bytes(64, 0, 128, 256) == 0
    lib.moe_row_map.argtypes = [P, P, P, I, I, I, P, P, P]
    assert lib.moe_row_map(fake, fake, fake, 8, 64, 2, fake, null, null) == -1
    assert lib.moe_row_map(fake, fake, fake, 300, 64, 2, fake, fake, null) == -1
    assert lib.moe_row_map(null, null, null, 8, 0, 2, null, null, null) == 0
    lib.moe_expert_ffn_fused_fwd.argtypes = [P, P, P, P, P, P, I, I, I, I, I, P, P, P, Z, P]
    fwd = lambda x, d, ws, n: lib.moe_expert_ffn_fused_fwd(x, fake, fake, fake, fake, fake, 64, 2, d, 8, 256, fake, fake, ws, Z(n), null)
    assert fwd(null, 128, fake, need) == -1
    assert fwd(fake, 120, fake, need) == -2          # d must be a multiple of 16
    assert fwd(fake, 128, fake, need - 1) == -3
    assert fwd(P(4100), 128, fake, need) == -2       # 16-byte alignment
    lib.moe_expert_ffn_fused_bwd.argtypes = [P, P, P, P, P, P, P, P, P, I, I, I, I, I, P, P, P, I, I, P, P, Z, P]
    bwd = lambda dy, gdt, dw, n: lib.moe_expert_ffn_fused_bwd(fake, dy, fake, fake, fake, fake, fake, fake, fake, 64, 2, 128, 8, 256,
                                                              fake, fake, fake, gdt, 0, dw, fake, Z(n), null)
    assert bwd(null, 0, fake, need) == -1
    assert bwd(fake, 2, fake, need) == -2            # weight gradients are fp32 or bf16
    assert bwd(fake, 0, null, need) == -1
    assert bwd(fake, 0, fake, need - 1) == -3


def test_stale_library_is_detected(monkeypatch):
    """The build stamps the library with a hash of its sources; a library from other sources is not current."""
    from paper_2505_11432_amd import build
    build.ensure_built()
    assert build.is_current()
    real = build.source_hash()
    monkeypatch.setattr(build, "source_hash", lambda: "0" * 64)
    assert not build.is_current()
    monkeypatch.undo()
    assert build.source_hash() == real and build.is_current()


def test_transpose_and_init_argument_errors(lib):
    P = ctypes.c_void_p
    fake, other = P(4096), P(8192)
    assert lib.moe_transpose(fake, 1, 1, 8, 8, fake, None) == -1          # in place is not supported
    assert lib.moe_transpose(None, 1, 1, 8, 8, other, None) == -1
    assert lib.moe_transpose(fake, 9, 1, 8, 8, other, None) == -2
    assert lib.moe_transpose(None, 1, 0, 8, 8, None, None) == 0


def test_ceilings_library_exports_its_header():
    """libmoe_ceilings.so (measurement aids of bench.py) exports every symbol include/moe_ceilings.h declares."""
    from paper_2505_11432_amd import build
    build.ensure_built()
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "moe_ceilings.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(moe_ceiling_[a-z0-9_]+)\s*\(", text)))
    assert names == ["moe_ceiling_copy", "moe_ceiling_mfma_lds_dma_loop", "moe_ceiling_mfma_lds_loop", "moe_ceiling_mfma_loop",
                     "moe_ceiling_read"]
    lib2 = ctypes.CDLL(build.CEILINGS_LIB_PATH)
    for n in names:
        assert hasattr(lib2, n), n
    assert lib2.moe_ceiling_copy(None, None, ctypes.c_size_t(16), None) == -1
    assert lib2.moe_ceiling_mfma_loop(0, None, 10, 1, None, None) == -1
    lib2.moe_ceiling_mfma_lds_dma_loop.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                                   ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    assert lib2.moe_ceiling_mfma_lds_dma_loop(None, None, 65536, 8, 7, 1, None, None) == -1
    one = ctypes.c_void_p(16)                  # never dereferenced: the argument checks come first
    assert lib2.moe_ceiling_mfma_lds_dma_loop(one, one, 65536, 6, 7, 1, one, None) == -1      # iters not a multiple of 4
    assert lib2.moe_ceiling_mfma_lds_dma_loop(one, one, 65536 + 16, 8, 7, 1, one, None) == -1  # src not whole 64 KiB slices
    assert lib2.moe_ceiling_mfma_lds_dma_loop(one, one, 65536, 8, 8, 1, one, None) == -1       # unknown flag


def test_profile_labels():
    from paper_2505_11432_amd.profile_summary import label
    base = "_ZN3moe4mfma23grouped_gemm_dma_kernelILi256ELi256ELi64ELi2ELi2ELi4ELNS0_6LayoutE1ELS2_1ELNS0_4ModeE1ELNS0_3EpiE0E"
    assert label(base + "fDF16bEEvNS0_4ArgsE") == "grouped_gemm<256x256x64 s2 w2x4 TN kseg store out=f32 in=bf16>"
    assert label(base.replace("LayoutE1ELS2_1E", "LayoutE0ELS2_0E").replace("ModeE1", "ModeE0").replace("EpiE0", "EpiE1")
                 + "DF16bhEEvNS0_4ArgsE") == "grouped_gemm<256x256x64 s2 w2x4 NT rowseg swiglu out=bf16 in=e4m3>"
    assert label("_ZN3moe12_GLOBAL__N_114combine_kernelIDF16bDF16bLi8ELi2EEEvPKT_") == "combine_kernel"
