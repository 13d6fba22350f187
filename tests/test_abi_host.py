"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device.
(The error paths return before any HIP call, so fake non-NULL pointers are safe.)"""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_1908_07782_amd as combo
    if not os.path.exists(combo.LIB_PATH):
        from paper_1908_07782_amd import build
        build.build()
    return combo.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "combo.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(combo_[a-z0-9_]+)\s*\(", header))
    assert {"combo_make_peer_table", "combo_segment_gossip_round",
            "combo_local_sgd_then_gossip", "combo_strerror"} <= declared
    for name in declared:
        assert hasattr(L, name), name


def test_no_torch_or_oracle_in_the_boundary():
    header = open(os.path.join(ROOT, "include", "combo.h")).read()
    assert "torch" not in header.lower() and "at::" not in header
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_1908_07782_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+\.*oracle", text, flags=re.M), f
                assert "combo_ref" not in text and "oracle/" not in text, f


def test_strerror_is_total(L):
    for code in range(-6, 2):
        s = L.combo_strerror(code)
        assert s and len(s) > 3


FAKE_A = ctypes.c_void_p(0x10000000)
FAKE_B = ctypes.c_void_p(0x20000000)
FAKE_C = ctypes.c_void_p(0x30000000)
FAKE_T = ctypes.c_void_p(0x40000000)
EINVAL, EALIAS, ERANGE = -1, -2, -3


def test_peer_table_argument_errors(L):
    f = L.combo_make_peer_table
    assert f(FAKE_T, 0, 1, 0, 0, 0, None) == EINVAL          # N < 1
    assert f(FAKE_T, 4, 0, 1, 0, 0, None) == EINVAL          # S < 1
    assert f(FAKE_T, 4, 2, -1, 0, 0, None) == EINVAL         # R < 0
    assert f(FAKE_T, 4, 2, 4, 0, 0, None) == EINVAL          # R > N-1
    assert f(None, 4, 2, 1, 0, 0, None) == EINVAL            # NULL table with R > 0
    assert f(None, 4, 2, 0, 0, 0, None) == 0                 # R == 0: empty table, nothing to do
    assert f(FAKE_T, 16385, 2, 1, 0, 0, None) == ERANGE      # LDS limit


def test_pooled_table_and_degree_argument_errors(L):
    f = L.combo_make_peer_table_pooled
    assert f(FAKE_T, 0, 1, 0, 0, 0, None) == EINVAL
    assert f(FAKE_T, 4, 2, 4, 0, 0, None) == EINVAL
    assert f(None, 4, 2, 1, 0, 0, None) == EINVAL
    assert f(None, 4, 2, 0, 0, 0, None) == 0
    assert f(FAKE_T, 16385, 2, 1, 0, 0, None) == ERANGE
    g = L.combo_peer_in_degree
    assert g(None, FAKE_T, 4, 2, 1, None) == EINVAL
    assert g(FAKE_A, None, 4, 2, 1, None) == EINVAL
    assert g(FAKE_A, FAKE_T, 0, 2, 1, None) == EINVAL
    assert g(FAKE_A, FAKE_T, 20000, 2, 1, None) == ERANGE


def test_dynamic_argument_errors(L):
    f = L.combo_make_peer_table_dynamic
    assert f(FAKE_T, None, 4, 2, 1, 0, 0, None) == EINVAL
    assert f(None, FAKE_C, 4, 2, 1, 0, 0, None) == EINVAL
    assert f(FAKE_T, FAKE_C, 4, 2, 4, 0, 0, None) == EINVAL
    assert f(FAKE_T, FAKE_C, 16385, 2, 1, 0, 0, None) == ERANGE
    assert f(None, None, 4, 2, 0, 0, 0, None) == 0
    g = L.combo_segment_gossip_round_dynamic
    assert g(FAKE_A, FAKE_B, 1024, FAKE_T, None, None, 4, 1000, 4, 2, None) == EINVAL
    assert g(FAKE_A, FAKE_A, 1024, FAKE_T, None, FAKE_C, 4, 1000, 4, 2, None) == EALIAS
    assert g(FAKE_A, FAKE_B, 999, FAKE_T, None, FAKE_C, 4, 1000, 4, 2, None) == EINVAL


def test_divergence_argument_errors(L):
    ws = L.combo_aggregation_divergence_workspace
    assert ws(0, 10) == EINVAL and ws(4, 0) == EINVAL and ws(1100, 1000) == ERANGE
    need = ws(32, 11_689_512)
    assert need == 4096 * 32 * 8
    assert ws(4, 100) == 4096 * 4 * 8
    f = L.combo_aggregation_divergence
    assert f(None, FAKE_B, 1024, None, 4, 1000, FAKE_C, 10**6, None) == EINVAL
    assert f(FAKE_A, FAKE_B, 999, None, 4, 1000, FAKE_C, 10**6, None) == EINVAL
    assert f(FAKE_A, FAKE_B, 1024, None, 4, 1000, None, 10**6, None) == EINVAL
    assert f(FAKE_A, FAKE_B, 1024, None, 4, 1000, FAKE_C, 8, None) == EINVAL
    assert f(FAKE_A, FAKE_B, 1024, None, 4, 1000, ctypes.c_void_p(0x30000004), 10**6, None) == EINVAL


def test_divergence_noalloc_argument_errors(L):
    f = L.combo_aggregation_divergence_noalloc
    f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p,
                  ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p]
    assert f(None, FAKE_B, 1024, 0, None, 4, 1000, None) == EINVAL
    assert f(FAKE_A, None, 1024, 0, None, 4, 1000, None) == EINVAL
    assert f(FAKE_A, FAKE_B, 999, 0, None, 4, 1000, None) == EINVAL       # ld < P
    assert f(FAKE_A, FAKE_B, 0, 100, None, 4, 1000, None) == EINVAL       # tile width not a power of two
    assert f(FAKE_A, FAKE_B, 1024, 0, None, 0, 1000, None) == EINVAL
    assert f(FAKE_A, FAKE_B, 1024, 0, None, 129, 1000, None) == ERANGE    # beyond the held array
    assert f(FAKE_A, FAKE_B, 1024, 0, None, 2000, 1000, None) == ERANGE
    header = open(os.path.join(ROOT, "include", "combo.h")).read()
    assert re.search(r"#define\s+COMBO_DIVERGENCE_NOALLOC_MAX_WORKERS\s+128\b", header)


def test_bandwidth_probe_argument_errors(L):
    f = L.combo_bandwidth_probe
    f.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
                  ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
    assert f(-1, FAKE_A, FAKE_B, 4, 1024, 1000, 0, 1, None) == EINVAL        # unknown kind
    assert f(7, FAKE_A, FAKE_B, 4, 1024, 1000, 0, 1, None) == EINVAL
    assert f(0, None, FAKE_B, 4, 1024, 1000, 0, 1, None) == EINVAL
    assert f(0, FAKE_A, None, 4, 1024, 1000, 0, 1, None) == EINVAL           # only the write probe needs no source
    assert f(0, FAKE_A, FAKE_B, 4, 999, 1000, 0, 1, None) == EINVAL          # ld < P
    assert f(0, FAKE_A, FAKE_B, 4, 1001, 1000, 0, 1, None) == EINVAL         # pitch not a multiple of 4
    assert f(0, ctypes.c_void_p(0x10000004), FAKE_B, 4, 1024, 1000, 0, 1, None) == EINVAL
    assert f(0, FAKE_A, FAKE_A, 4, 1024, 1000, 0, 1, None) == EALIAS
    assert f(0, FAKE_A, FAKE_B, 4, 1 << 61, 1000, 0, 1, None) == ERANGE


def test_hashed_round_argument_errors(L):
    f = L.combo_round_hashed

    def call(dst=FAKE_A, src=FAKE_B, grads=None, tau=0, ld=1024, tile=0, N=4, P=1000, S=4, R=2):
        return f(dst, src, grads, tau, ctypes.c_float(0.1), ld, tile, None, N, P, S, R, 1, 2, None)

    assert call(R=4) == EINVAL and call(S=0) == EINVAL and call(dst=None) == EINVAL
    assert call(tau=1) == EINVAL                    # gradients missing
    assert call(tau=-1) == EINVAL
    assert call(ld=999) == EINVAL
    assert call(tile=100) == EINVAL
    assert call(N=20, R=9) == ERANGE                # in-kernel draw supports R <= 8
    assert call(ld=1001, P=1001) == ERANGE          # pitch not a multiple of 4
    assert call(dst=ctypes.c_void_p(0x10000004)) == ERANGE
    assert call(N=300, R=2) == ERANGE               # slab does not fit
    assert call(dst=FAKE_B) == EALIAS
    assert call(grads=FAKE_B, tau=1) == EALIAS


def test_round_argument_errors(L):
    f = L.combo_segment_gossip_round
    ok = dict(N=4, P=1000, S=4, R=2, ld=1024)

    def call(dst=FAKE_A, src=FAKE_B, peers=FAKE_T, d=None, **kw):
        a = dict(ok, **kw)
        return f(dst, src, a["ld"], peers, d, a["N"], a["P"], a["S"], a["R"], None)

    assert call(N=0) == EINVAL
    assert call(S=0) == EINVAL
    assert call(S=1001) == EINVAL                 # more segments than parameters
    assert call(R=-1) == EINVAL
    assert call(R=4) == EINVAL                    # needs R <= N-1
    assert call(ld=999) == EINVAL                 # pitch shorter than a row
    assert call(dst=None) == EINVAL
    assert call(src=None) == EINVAL
    assert call(peers=None) == EINVAL
    assert call(dst=FAKE_A, src=FAKE_A) == EALIAS
    # back buffer starting inside the front buffer (4 rows x 1024 floats = 16 KiB)
    assert call(dst=ctypes.c_void_p(0x20000000 + 4 * 1024 * 4 - 4), src=FAKE_B) == EALIAS
    assert call(dst=ctypes.c_void_p(0x20000000 - 4 * 1024 * 4 + 4), src=FAKE_B) == EALIAS
    # grid limit: N * ceil(P / tile) must stay below 2^31
    low = ctypes.c_void_p(0x1000)                 # a table below the (huge) back buffer
    assert f(FAKE_A, ctypes.c_void_p(0x7000000000000000), 1 << 40, low, None, 16384, 1 << 40, 4, 2,
             None) == ERANGE
    # the table, the dataset sizes (and the status array) must not lie inside the back buffer
    assert call(peers=ctypes.c_void_p(0x10000000 + 64)) == EALIAS
    assert call(d=ctypes.c_void_p(0x10000000 + 4 * 1024 * 4 - 4)) == EALIAS
    g = L.combo_segment_gossip_round_dynamic
    assert g(FAKE_A, FAKE_B, 1024, FAKE_T, None, ctypes.c_void_p(0x10000000 + 100), 4, 1000, 4, 2, None) == EALIAS
    # N * ld * 4 beyond 64 bits
    assert f(FAKE_A, FAKE_B, 1 << 61, low, None, 8, 1000, 4, 2, None) == ERANGE


def test_relayout_argument_errors(L):
    f = L.combo_round_relayout
    f.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int64,
                  ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_void_p,
                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                  ctypes.c_int32, ctypes.c_void_p]

    def call(dst=FAKE_A, dst_ld=1024, dst_tile=0, src=FAKE_B, src_ld=1024, src_tile=64, grads=None, tau=0,
             peers=FAKE_T, status=None, N=4, P=1000, S=4, R=2):
        return f(dst, dst_ld, dst_tile, src, src_ld, src_tile, grads, tau, 0.1, peers, None, status, N, P, S,
                 R, None)

    assert call(N=0) == EINVAL and call(S=1001) == EINVAL and call(R=4) == EINVAL
    assert call(dst=None) == EINVAL and call(src=None) == EINVAL and call(peers=None) == EINVAL
    assert call(tau=1) == EINVAL and call(tau=-1) == EINVAL
    assert call(src_tile=100) == EINVAL and call(dst_tile=7) == EINVAL
    assert call(dst_ld=999) == EINVAL                               # row-major side: pitch below P
    assert call(src_tile=0, src_ld=999) == EINVAL
    assert call(dst_tile=128) == ERANGE                             # two tiled sides of different widths
    assert call(dst_ld=1001, P=1001, S=4) == ERANGE                 # pitch not a multiple of 4
    assert call(dst=ctypes.c_void_p(0x10000004)) == ERANGE          # not 16-byte aligned
    assert call(N=300, R=2, src_tile=64) == ERANGE                  # slab does not fit
    assert call(status=FAKE_C, grads=FAKE_C, tau=1) == ERANGE
    assert call(dst=FAKE_B) == EALIAS
    assert call(grads=FAKE_B, tau=1) == EALIAS
    assert call(peers=ctypes.c_void_p(0x10000000 + 16)) == EALIAS


def test_fused_argument_errors(L):
    f = L.combo_local_sgd_then_gossip

    def call(dst=FAKE_A, src=FAKE_B, grad=FAKE_C, peers=FAKE_T, N=4, P=1000, S=4, R=2, ld=1024):
        return f(dst, src, grad, ctypes.c_float(0.01), ld, peers, None, N, P, S, R, None)

    assert call(grad=None) == EINVAL
    assert call(grad=FAKE_B) == EALIAS
    assert call(grad=FAKE_A) == EALIAS
    assert call(dst=FAKE_B) == EALIAS
    assert call(R=9) == EINVAL


def test_tiled_layout_sizes_and_recommended_widths(L):
    """Pure host arithmetic: which tile width the library recommends and how many floats a
    tiled matrix has."""
    cols, elems = L.combo_tiled_cols, L.combo_tiled_elems
    assert cols(0, 1) == EINVAL and cols(4, -1) == EINVAL
    # the narrowest width whose tile reaches 8 KiB: 8 KiB for powers of two, up to 16 KiB between
    assert [cols(n, 4) for n in (4, 8, 16, 32)] == [512, 256, 128, 64] and cols(2, 1) == 1024
    assert [cols(n, 2) for n in (3, 5, 10, 12, 20, 24, 30)] == [1024, 512, 256, 256, 128, 128, 128]
    assert cols(1, 0) == 1024
    # more than 8 replicas: the widest tile within 32 KiB
    assert [cols(n, 12) for n in (16, 20, 30, 32, 40, 64)] == [512, 256, 256, 256, 128, 128]
    # then the widest of 64, 32, 16, 8 columns whose tile stays within 32 KiB
    assert [cols(n, 3) for n in (33, 100, 128, 129, 256, 257, 512, 513, 1000)] == \
        [64, 64, 64, 32, 32, 16, 16, 8, 8]
    assert cols(1000, 5) == 8 and cols(1000, 6) == ERANGE and cols(3000, 2) == ERANGE
    assert elems(4, 1000, 64) == 16 * 4 * 64 and elems(7, 63, 8) == 8 * 7 * 8
    assert elems(4, 1000, 4) == EINVAL and elems(4, 1000, 100) == EINVAL and elems(4, 1000, 2048) == EINVAL
    assert elems(0, 1000, 64) == EINVAL and elems(4, 0, 64) == EINVAL


def test_tuning_knobs(L):
    assert L.combo_get_tune(0) == 0                  # row-tile width: automatic
    assert L.combo_tune(0, 1000) == EINVAL
    assert L.combo_tune(99, 1) == EINVAL
    old = L.combo_get_tune(0)
    for v in (1024, 2048, 4096):
        assert L.combo_tune(0, v) == 0 and L.combo_get_tune(0) == v
    assert L.combo_tune(0, old) == 0
    assert L.combo_get_tune(1) in (0, 1)
    assert L.combo_get_tune(77) == EINVAL
    assert L.combo_tune(3, 3) == EINVAL and L.combo_tune(3, 2) == 0 and L.combo_tune(3, 0) == 0
    assert L.combo_tune(4, 100) == EINVAL and L.combo_tune(4, 2048) == EINVAL
    assert L.combo_tune(4, 128) == 0 and L.combo_get_tune(4) == 128 and L.combo_tune(4, 0) == 0
    assert L.combo_tune(2, 2) == EINVAL and L.combo_tune(2, 1) == 0 and L.combo_tune(2, 0) == 0


def test_header_is_plain_c(tmp_path):
    """include/combo.h must compile as C99 (no C++ or HIP types in the boundary) and a C
    translation unit that takes the address of every declared function must link against
    the shared library."""
    import subprocess
    import paper_1908_07782_amd as combo
    header = open(os.path.join(ROOT, "include", "combo.h")).read()
    names = sorted(set(re.findall(r"\b(combo_[a-z0-9_]+)\s*\(", re.sub(r"/\*.*?\*/", "", header, flags=re.S))))
    src = tmp_path / "use_combo.c"
    src.write_text('#include "combo.h"\n#include <stdio.h>\ntypedef void (*fn)(void);\nint main(void) {\n  fn f[] = {'
                   + ", ".join(f"(fn){n}" for n in names)
                   + '};\n  printf("%d symbols %s\\n", (int)(sizeof f / sizeof f[0]), combo_strerror(COMBO_EALIAS));\n'
                     "  return combo_tune(99, 0) == COMBO_EINVAL ? 0 : 1;\n}\n")
    exe = tmp_path / "use_combo"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), combo.LIB_PATH, "-Wl,-rpath," + os.path.dirname(combo.LIB_PATH),
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stdout + out.stderr
    assert f"{len(names)} symbols" in out.stdout
