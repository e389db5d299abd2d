"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side argument checks return error codes (never abort) before any GPU work."""
import ctypes
import os
import re

import pytest

from paper_2503_13565_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mxfp4.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(mxfp4_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    names = declared_functions()
    assert len(names) >= 12
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names
    assert binding.version().startswith("mxfp4-gfx950")


def test_product_never_touches_the_oracle():
    # the product package must not import the test oracle
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2503_13565_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", src, flags=re.M), f
                assert "liboracle" not in src, f


P16 = ctypes.c_void_p(4096)          # a non-NULL, 16-byte aligned fake pointer; never dereferenced on error paths
P2 = ctypes.c_void_p(4098)


@pytest.mark.parametrize("args,code", [
    ((None, -1, 32, 32, None, None, None), 2),                 # N < 0
    ((P16, 4, 48, 48, P16, P16, None), 2),                      # K % 32
    ((P16, 4, 64, 32, P16, P16, None), 2),                      # ldw < K
    ((None, 4, 64, 64, P16, P16, None), 1),                     # NULL input
    ((P2, 4, 64, 64, P16, P16, None), 3),                       # misaligned input
    ((P16, 4, 64, 68, P16, P16, None), 3),                      # ldw % 8
    ((P16, 0, 64, 64, None, None, None), 0),                    # N == 0 is a no-op
])
def test_direct_cast_argument_checks(args, code):
    lib = binding.load()
    assert lib.mxfp4_direct_cast(*args) == code
    if code:
        assert lib.mxfp4_last_error()


@pytest.mark.parametrize("args,code", [
    ((None, 1, 64, P16, P16, 8, 64, P16, 8, None), 1),          # x NULL
    ((P16, 1, 64, None, P16, 8, 64, P16, 8, None), 1),          # q NULL
    ((P16, 0, 64, P16, P16, 8, 64, P16, 8, None), 2),           # M < 1
    ((P16, 1, 64, P16, P16, 0, 64, P16, 8, None), 2),           # N < 1
    ((P16, 1, 64, P16, P16, 8, 40, P16, 8, None), 2),           # K % 32
    ((P16, 1, 64, P16, P16, 8, 131072, P16, 8, None), 2),       # K too large
    ((P16, 1, 32, P16, P16, 8, 64, P16, 8, None), 2),           # ldx < K
    ((P2, 1, 64, P16, P16, 8, 64, P16, 8, None), 3),            # x misaligned
    ((P16, 1, 64, P2, P16, 8, 64, P16, 8, None), 3),            # q misaligned
    ((P16, 2, 68, P16, P16, 8, 64, P16, 8, None), 3),           # ldx % 8
])
def test_gemm_argument_checks(args, code):
    lib = binding.load()
    assert lib.mxfp4_woq_gemm(*args) == code
    assert lib.mxfp4_last_error()


def test_argmax_workspace_size_and_checks():
    lib = binding.load()
    need = lib.mxfp4_woq_gemm_argmax_workspace_bytes(4, 32000, 4096)
    assert need >= 4 * 8 and need % 8 == 0
    assert lib.mxfp4_woq_gemm_argmax_workspace_bytes(0, 1, 32) == 0
    # bad K is reported before the workspace is looked at
    assert lib.mxfp4_woq_gemm_argmax(P16, 1, 64, P16, P16, 8, 40, P16, None, None, 0, None) == 2


P1 = ctypes.c_void_p(4097)


@pytest.mark.parametrize("bias,act,res,ldr,n,code", [
    (None, 7, None, 0, 8, 6),             # unknown act
    (None, 1, None, 0, 9, 2),             # the gate needs an even N
    (None, 0, P16, 4, 8, 2),              # ldr < N
    (None, 1, P16, 3, 8, 2),              # ldr < N / 2 with the gate
    (P1, 0, None, 0, 8, 3),               # bias not 2-byte aligned
    (None, 0, P1, 8, 8, 3),               # residual not 2-byte aligned
])
def test_fused_argument_checks(bias, act, res, ldr, n, code):
    lib = binding.load()
    rc = lib.mxfp4_woq_gemm_fused(P16, 1, 64, P16, P16, n, 64, bias, act, res, ldr, P16, 8, None, 0, 0, None)
    assert rc == code and lib.mxfp4_last_error()


def test_fused_refuses_paths_without_a_fused_form():
    lib = binding.load()
    for path in (binding.PATH_VALU_BITS, binding.PATH_VALU_LUT):
        assert lib.mxfp4_woq_gemm_fused(P16, 1, 64, P16, P16, 8, 64, None, 0, None, 0, P16, 8, None, 0, path,
                                        None) == 6


def test_tile_repack_sizes_and_checks():
    lib = binding.load()
    # whole tiles of 16 rows; whole items of four steps of 128 elements
    assert lib.mxfp4_tile_repack_q_bytes(17, 256) == 32 * 128
    assert lib.mxfp4_tile_repack_s_bytes(17, 256) == 2 * 1 * 256
    assert lib.mxfp4_tile_repack_s_bytes(16, 11008) == 22 * 256
    assert lib.mxfp4_tile_repack(P16, P16, 16, 96, P16, P16, None) == 2        # K % 128
    assert lib.mxfp4_tile_repack(None, P16, 16, 128, P16, P16, None) == 1
    assert lib.mxfp4_tile_repack(P16, P16, 16, 128, None, P16, None) == 1
    assert lib.mxfp4_tile_repack(P16, P16, 16, 128, P2, P16, None) == 3
    assert lib.mxfp4_woq_gemm_tiled(P16, 1, 128, P16, P2, 16, 128, P16, 16, None) == 3     # s_tiled alignment
    assert lib.mxfp4_woq_gemm_tiled(P16, 1, 96, P16, P16, 16, 96, P16, 16, None) == 2      # K % 128


@pytest.mark.parametrize("args,code", [
    ((P16, 4, 48, 48, P16, P16, None), 2),                      # K % 32
    ((P16, 4, 64, 32, P16, P16, None), 2),                      # ldw < K
    ((None, 4, 64, 64, P16, P16, None), 1),
    ((P16, 4, 64, 64, P2, P16, None), 3),                       # q8 not 8-byte aligned
    ((P16, 0, 64, 64, None, None, None), 0),                    # N == 0 is a no-op
])
def test_e4m3_cast_argument_checks(args, code):
    lib = binding.load()
    assert lib.mxfp4_e4m3_direct_cast(*args) == code
    assert lib.mxfp4_e4m3_direct_cast_bits(*args) == code


def test_e4m3_product_argument_checks():
    lib = binding.load()
    assert lib.mxfp4_e4m3_woq_gemm(None, 1, 64, P16, P16, 8, 64, P16, 8, None) == 1
    assert lib.mxfp4_e4m3_woq_gemm(P16, 1, 64, P2, P16, 8, 64, P16, 8, None) == 3          # q8 alignment
    assert lib.mxfp4_e4m3_woq_gemm(P16, 1, 64, P16, P16, 8, 40, P16, 8, None) == 2         # K % 32
    assert lib.mxfp4_e4m3_woq_gemm(P16, 1, 64, P16, P16, 1 << 20, 4096, P16, 8, None) == 2  # N * K beyond 2 GiB
    assert lib.mxfp4_e4m3_dequant(P16, P16, 4, 64, None, 64, None) == 1


@pytest.mark.parametrize("args,code", [
    ((P16, 4, 48, 48, P16, P16, None), 2),                      # K % 32
    ((P16, 4, 64, 32, P16, P16, None), 2),                      # ldw < K
    ((None, 4, 64, 64, P16, P16, None), 1),
    ((P16, 4, 64, 64, P2, P16, None), 3),                       # q6 not 8-byte aligned
    ((P16, 0, 64, 64, None, None, None), 0),                    # N == 0 is a no-op
])
def test_e2m3_cast_argument_checks(args, code):
    lib = binding.load()
    assert lib.mxfp4_e2m3_direct_cast(*args) == code
    assert lib.mxfp4_e2m3_direct_cast_bits(*args) == code


def test_e2m3_product_argument_checks():
    lib = binding.load()
    assert lib.mxfp4_e2m3_woq_gemm(None, 1, 128, P16, P16, 8, 128, P16, 8, None) == 1
    assert lib.mxfp4_e2m3_woq_gemm(P16, 1, 128, P2, P16, 8, 128, P16, 8, None) == 3          # q6 alignment
    assert lib.mxfp4_e2m3_woq_gemm(P16, 1, 64, P16, P16, 8, 40, P16, 8, None) == 2           # K % 32
    assert lib.mxfp4_e2m3_woq_gemm(P16, 1, 4096, P16, P16, 1 << 20, 4096, P16, 8, None) == 2  # beyond 2 GiB
    assert lib.mxfp4_e2m3_dequant(P16, P16, 4, 64, None, 64, None) == 1


def _desc(**kw):
    d = binding.GemmDesc()
    base = dict(x_bf16=P16.value, M=1, ldx=64, q_packed=P16.value, scales_e8m0=P16.value, N=8, K=64,
                bias_bf16=None, residual_bf16=None, ldr=0, y_bf16=P16.value, ldy=8, argmax_out=None, max_out=None,
                act=0, flags=0)
    base.update(kw)
    for name, v in base.items():
        setattr(d, name, v)
    return d


def test_grouped_descriptor_matches_the_header():
    # 14 eight-byte fields and two 32-bit ones, no padding
    assert ctypes.sizeof(binding.GemmDesc) == 14 * 8 + 8
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    body = re.search(r"typedef struct mxfp4_gemm_desc \{(.*?)\} mxfp4_gemm_desc;", text, flags=re.S).group(1)
    fields = re.findall(r"(\w+);", body)
    assert fields == [name for name, _ in binding.GemmDesc._fields_]


@pytest.mark.parametrize("kw,code", [
    (dict(K=40), 2),                          # K % 32
    (dict(x_bf16=None), 1),
    (dict(flags=6), 6),
    (dict(act=9), 6),
    (dict(act=1, N=7, ldy=4), 2),             # the gate needs an even N
    (dict(residual_bf16=P16.value, ldr=4), 2),
    (dict(argmax_out=P16.value), 6),          # the pick takes no y
    (dict(argmax_out=P16.value, y_bf16=None, act=1), 6),
    (dict(argmax_out=P16.value, y_bf16=None, K=40), 2),
])
def test_grouped_argument_checks_name_the_descriptor(kw, code):
    # (without a GPU a valid descriptor ends at the device query, so the bad one stands first)
    lib = binding.load()
    descs = (binding.GemmDesc * 2)(_desc(**kw), _desc())
    assert lib.mxfp4_woq_gemm_grouped(descs, 2, None, 0, None) == code
    assert lib.mxfp4_last_error().decode().startswith("descriptor 0: ")


def test_grouped_trivial_cases():
    lib = binding.load()
    assert lib.mxfp4_woq_gemm_grouped(None, 0, None, 0, None) == 0
    assert lib.mxfp4_woq_gemm_grouped(None, 2, None, 0, None) == 1
    assert lib.mxfp4_woq_gemm_grouped(None, -1, None, 0, None) == 2
    assert lib.mxfp4_woq_gemm_grouped_workspace_bytes(None, 3) == 0
    descs = (binding.GemmDesc * 2)(_desc(M=16, N=4096, K=28672), _desc(M=1, N=4096, K=4096))
    assert lib.mxfp4_woq_gemm_grouped_workspace_bytes(descs, 2) == lib.mxfp4_woq_gemm_workspace_bytes(16, 4096, 28672) > 0
