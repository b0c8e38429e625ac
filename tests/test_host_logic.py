"""CPU checks of the library's host-side pieces: the tile enumeration / classification header the
kernels compile (brute-forced on the host), and that the built C-ABI library exports every symbol
include/hstu_attn.h declares.  No kernel is launched here."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_16986_amd", "csrc")


@pytest.fixture(scope="module")
def geom(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("geom") / "libgeometry_check.so")
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", so,
                           os.path.join(CSRC, "geometry_check.cpp")])
    lib = ctypes.CDLL(so)
    lib.geometry_check.restype = ctypes.c_int
    lib.geometry_check.argtypes = [ctypes.c_int] * 6
    return lib


CASES = [(L, M, K1, K2) for L in (1, 31, 64, 65, 200, 333)
         for (M, K1, K2) in ((0, -1, 0), (0, 40, 10), (0, 1, 0), (0, 0, 70), (0, 0, 0), (0, 64, 64), (0, 100, 33),
                             (7, -1, 0), (7, 50, 20), (64, 33, 3), (10 ** 9, 10, 5), (5, 0, 40), (1, 500, 0))]


@pytest.mark.parametrize("block_rows,BN", [(256, 64), (128, 64), (128, 32), (32, 32)])
def test_tile_enumeration_and_classification(geom, block_rows, BN):
    for L, M, K1, K2 in CASES:
        M = min(M, L)
        rc = geom.geometry_check(L, M, K1, K2, block_rows, BN)
        assert rc == 0, f"property {rc} violated for L={L} M={M} K1={K1} K2={K2} rows={block_rows} BN={BN}"


def test_tile_enumeration_random(geom):
    rng = np.random.default_rng(0)
    for _ in range(300):
        L = int(rng.integers(1, 700))
        M = int(rng.integers(0, L + 1)) if rng.random() < 0.5 else 0
        K1 = int(rng.choice([-1, 0, 1, 5, 63, 64, 65, 130, 1000]))
        K2 = int(rng.choice([0, 1, 31, 64, 100, 1000]))
        br, bn = [(256, 64), (128, 64), (128, 32)][int(rng.integers(0, 3))]
        rc = geom.geometry_check(L, M, K1, K2, br, bn)
        assert rc == 0, f"property {rc} violated for L={L} M={M} K1={K1} K2={K2} rows={br} BN={bn}"


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "hstu_attn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(hstu_[a-z_]+)\s*\(", header))
    assert {"hstu_attn_fwd", "hstu_attn_bwd", "hstu_gated_norm_fwd", "hstu_gated_norm_bwd"} <= declared
    lib_path = os.path.join(ROOT, "paper_2602_16986_amd", "libhstu_attn.so")
    if not os.path.exists(lib_path):
        from paper_2602_16986_amd.build import build_library
        build_library()
    lib = ctypes.CDLL(lib_path)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in hstu_attn.h but not exported"
    lib.hstu_status_string.restype = ctypes.c_char_p
    assert lib.hstu_status_string(0) == b"HSTU_OK"
    assert b"WORKSPACE" in lib.hstu_status_string(-4)


def test_flop_accounting_matches_oracle_pair_count():
    from oracle import hstu_oracle as orc
    from paper_2602_16986_amd import flops
    rng = np.random.default_rng(1)
    for _ in range(200):
        L = int(rng.integers(0, 300))
        M = int(rng.integers(0, L + 1)) if rng.random() < 0.5 else 0
        K1 = int(rng.choice([-1, 0, 1, 2, 17, 64, 1000]))
        K2 = int(rng.choice([0, 1, 9, 64, 1000]))
        assert flops.visible_pairs_one(L, M, K1, K2) == orc.count_pairs([L], [M], K1, K2), (L, M, K1, K2)
    from paper_2602_16986_amd import workloads as wl
    w = wl.config("C1")
    assert flops.attention_flops(w)["pairs"] == 62278


def test_workspace_query_rejects_descriptions_the_kernels_cannot_address():
    """hstu_attn_workspace_bytes returns 0 for an invalid description (no GPU call involved): the kernels
    address a tile row as sequence base + 32-bit byte offset built from a 24-bit row and a 24-bit stride."""
    from paper_2602_16986_amd import binding as hb
    lib = hb._lib

    def ws(**over):
        p = hb.HstuAttnParams()
        p.batch, p.num_heads, p.head_dim, p.total_tokens, p.max_seqlen, p.dtype = 2, 4, 128, 1000, 600, 0
        p.row_stride_q = p.row_stride_k = p.row_stride_v = p.row_stride_o = 4 * 128
        p.seq_offsets = 256                      # any non-null value: never dereferenced by the size query
        p.local_window, p.global_prefix, p.alpha, p.inv_n = -1, 0, 1.0, 1.0
        for k, v in over.items():
            setattr(p, k, v)
        return int(lib.hstu_attn_workspace_bytes(ctypes.byref(p), 0))

    assert ws() > 0
    assert ws(max_seqlen=1 << 24) == 0                       # row index must fit 24 bits
    assert ws(row_stride_k=1 << 23) == 0                     # 2^23 bf16 elements = 16 MiB per row
    assert ws(max_seqlen=1 << 20, row_stride_v=4096) == 0    # 2^20 rows x 8 KiB >= 4 GiB
    assert ws(row_stride_q=4 * 128 + 4) == 0                 # rows must start on 16-byte boundaries
    assert ws(head_dim=96) == 0


def test_public_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (and as C++) on its own, with no HIP or torch types."""
    import subprocess
    src = tmp_path / "abi.c"
    src.write_text('#include "hstu_attn.h"\nint main(void) { hstu_attn_params p; hstu_layer_params q; (void)p; (void)q; return 0; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)], check=True)
