"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates arguments before touching the device, and its kernel-selection
logic behaves."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2502_08145_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "axonn_linear.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(axonn_[a-z_0-9]+)\s*\(", src)))


def test_header_declares_the_three_entry_points():
    names = declared_functions()
    for n in ("axonn_linear_fwd", "axonn_linear_bwd_data", "axonn_linear_bwd_weight"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in declared_functions():
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"
    assert sorted(B.EXPORTS) == declared_functions()


def test_version_and_status_strings():
    assert B.version() >= 100
    assert B.status_string(0) == "ok"
    for code in (-1, -2, -3):
        assert B.status_string(code) not in ("ok", "unknown status")
    assert B.status_string(-99) == "unknown status"


ALIGNED = 0x1000  # never dereferenced: every call below must fail validation first


@pytest.mark.parametrize("fn", ["axonn_linear_fwd", "axonn_linear_bwd_data", "axonn_linear_bwd_weight"])
def test_invalid_arguments_are_refused_before_any_launch(fn):
    f = getattr(B, fn)
    bad = B.AXONN_ERR_INVALID_ARG
    kw = dict(stream=0, check=False)
    assert f(-1, 8, 8, "NN", ALIGNED, ALIGNED, ALIGNED, **kw) == bad
    assert f(8, -1, 8, "NN", ALIGNED, ALIGNED, ALIGNED, **kw) == bad
    assert f(8, 8, -1, "NN", ALIGNED, ALIGNED, ALIGNED, **kw) == bad
    assert f(2 ** 31, 8, 8, "NN", ALIGNED, ALIGNED, ALIGNED, **kw) == bad
    assert f(8, 8, 8, 3, ALIGNED, ALIGNED, ALIGNED, **kw) == bad
    assert f(8, 8, 8, -1, ALIGNED, ALIGNED, ALIGNED, **kw) == bad
    assert f(8, 8, 8, "NN", 0, ALIGNED, ALIGNED, **kw) == bad
    assert f(8, 8, 8, "NN", ALIGNED, 0, ALIGNED, **kw) == bad
    assert f(8, 8, 8, "NN", ALIGNED, ALIGNED, 0, **kw) == bad
    assert f(8, 8, 8, "NN", ALIGNED + 2, ALIGNED, ALIGNED, **kw) == bad
    assert f(8, 8, 8, "NN", ALIGNED, ALIGNED + 8, ALIGNED, **kw) == bad
    assert f(8, 8, 8, "NN", ALIGNED, ALIGNED, ALIGNED + 4, **kw) == bad
    assert f(8, 8, 8, "NN", ALIGNED, ALIGNED, ALIGNED, fp32_accumulate=2, **kw) == bad
    # an empty output is fine and touches nothing
    assert f(0, 8, 8, "NT", 0, 0, 0, **kw) == B.AXONN_OK
    assert f(8, 0, 8, "TN", 0, 0, 0, **kw) == B.AXONN_OK
    with pytest.raises(B.AxonnError):
        f(8, 8, 8, "NN", 0, 0, 0, stream=0)


def test_variant_table_and_selection():
    n = B.num_variants()
    assert n >= 2 and B.variant_name(0) == "naive"
    assert B.variant_name(n) is None and B.variant_name(-1) is None
    names = [B.variant_name(v) for v in range(n)]
    assert len(set(names)) == n
    # the guarded kernels take everything (the MFMA one wants K >= 1), tile kernels only whole tiles
    edge = names.index("mfma16_edge_128x128")
    assert edge == n - 1
    for lay in ("NN", "NT", "TN"):
        assert B.variant_supports(0, 3, 5, 7, lay) and B.variant_supports(0, 256, 256, 0, lay)
        assert B.variant_supports(edge, 3, 5, 7, lay) and B.variant_supports(edge, 1024, 1024, 1024, lay)
        assert not B.variant_supports(edge, 256, 256, 0, lay)
        for v in range(1, edge):
            assert not B.variant_supports(v, 100, 200, 300, lay)
            if names[v].startswith(("mfma16k64_256x128", "mfma16k64_128x256")) and lay != "NT":
                assert not B.variant_supports(v, 1024, 1024, 64 * 840, lay)  # the half tiles with 64-k stages: NT only
                continue
            assert B.variant_supports(v, 1024, 1024, 64 * 840, lay)          # 840 = lcm(1..8) K ranges
            assert not B.variant_supports(v, 1024, 1024, 1000, lay)
            assert not B.variant_supports(v, 1024, 1024, 200, lay)     # K must be a multiple of 64
            assert not B.variant_supports(v, 1024, 1024, 64 * 5 + 32, lay)
            assert not B.variant_supports(v, 1024, 1024, 64, lay)      # and long enough to fill the LDS buffers
            tail = names[v].rsplit("_", 1)[-1]
            splits = int(tail[2:]) if tail.startswith("sk") else 1
            assert B.variant_supports(v, 256, 256, 256 * splits, lay)   # per K range
            assert names[v].startswith("mfma16")                        # one MFMA shape: 16x16x32, K taken 64 at a time
            assert B.variant_supports(v, 256, 256, 256 * splits + 64 * splits, lay)
            assert not B.variant_supports(v, 256, 256, 256 * splits + 32, lay)
            # split-K keeps (splits - 1) fp32 partial tiles per output tile in a 64 MiB scratch area
            # with 1023 flags
            bm, bn = (int(x) for x in names[v].split("_")[1].split("x"))
            slots = (4096 // bm) * (4096 // bn) * (splits - 1)
            assert B.variant_supports(v, 4096, 4096, 4096, lay) == (slots <= 1023 and slots * bm * bn * 4 <= 64 << 20)
        # ragged or degenerate shapes go to the guarded kernel, large ones to an MFMA kernel
        assert B.select_variant(100, 200, 300, lay) == edge
        assert B.select_variant(1024, 1024, 1000, lay) == edge
        assert B.select_variant(256, 256, 0, lay) == 0
        for shape in [(2048, 12288, 4096), (4096, 16384, 2048), (8192, 8192, 8192), (2048, 8192, 2048)]:
            v = B.select_variant(*shape, lay)
            assert v > 0 and B.variant_supports(v, *shape, lay)
    assert B.select_variant(-1, 8, 8, "NN") == B.AXONN_ERR_INVALID_ARG
    # few tiles and a long K: split-K, unless it is switched off
    for lay in ("NN", "NT", "TN"):
        assert "_sk" in names[B.select_variant(2048, 4096, 16384, lay)]
        assert B.axonn_linear_set_split_k(False) is True
        assert "_sk" not in names[B.select_variant(2048, 4096, 16384, lay)]
        assert B.axonn_linear_set_split_k(True) is False
        assert "_sk" not in names[B.select_variant(8192, 8192, 8192, lay)]
    with pytest.raises(B.AxonnError):
        B.force_variant(n)
    B.force_variant(-1)


def test_workspace_queries_are_host_only():
    # split-K problems need 4 KiB of flags plus one fp32 tile per (tile, extra K range)
    assert B.axonn_linear_workspace_bytes(2048, 4096, 16384, "NT") == 4096 + 128 * 256 * 256 * 4
    assert B.axonn_linear_workspace_bytes(2048, 2048, 32768, "NN") == 4096 + 64 * 3 * 256 * 256 * 4
    assert B.axonn_linear_workspace_bytes(8192, 8192, 8192, "TN") == 0
    assert B.axonn_linear_workspace_bytes(100, 200, 300, "NN") == 0
    assert B.axonn_linear_workspace_bytes(0, 8, 8, "NN") == 0
    # a plan of 128 x 128 tiles with few slots: never less than what set_workspace accepts
    assert "128x128_sk" in B.plan_name(128, 128, 8192, "NT")
    assert B.axonn_linear_workspace_bytes(128, 128, 8192, "NT") == 4096 + 256 * 256 * 4
    # without a GPU no area can be registered: a call made now would run without split-K
    assert "_sk" in B.plan_name(2048, 4096, 16384, "NT") and "_sk" not in B.plan_name(2048, 4096, 16384, "NT", now=True)
    assert B.plan_name(8192, 8192, 8192, "TN", now=True) == B.plan_name(8192, 8192, 8192, "TN")
    L = B.lib()
    assert L.axonn_linear_set_workspace(0x1000, 0) == B.AXONN_ERR_INVALID_ARG      # pointer without size
    assert L.axonn_linear_set_workspace(None, 4096) == B.AXONN_ERR_INVALID_ARG     # size without pointer
    assert L.axonn_linear_set_workspace(0x1010, 1 << 20) == B.AXONN_ERR_INVALID_ARG  # not 256-byte aligned
    assert "scratch" in B.status_string(B.AXONN_ERR_WORKSPACE)


def test_transpose_arguments_are_checked_before_any_launch():
    f = lambda *a: B.axonn_transpose_bf16(*a, stream=0, check=False)
    bad = B.AXONN_ERR_INVALID_ARG
    assert f(-1, 8, ALIGNED, ALIGNED + (1 << 20)) == bad
    assert f(8, -1, ALIGNED, ALIGNED + (1 << 20)) == bad
    assert f(8, 8, 0, ALIGNED) == bad
    assert f(8, 8, ALIGNED, 0) == bad
    assert f(8, 8, ALIGNED + 1, ALIGNED + (1 << 20)) == bad          # odd address
    assert f(8, 8, ALIGNED, ALIGNED + 64) == bad                     # overlapping buffers
    assert f(1 << 31, 8, ALIGNED, ALIGNED + (1 << 20)) == bad
    assert f(0, 8, 0, 0) == B.AXONN_OK and f(8, 0, 0, 0) == B.AXONN_OK


def test_tuner_host_side():
    B.axonn_linear_tune_reset()
    assert B.axonn_linear_tuned("fwd", 256, 256, 256) is None
    with pytest.raises(B.AxonnError):
        B.axonn_linear_tuned(3, 256, 256, 256)
    # bad arguments are refused before anything touches a GPU
    res = B.TuneResult()
    L = B.lib()
    import ctypes
    bad = B.AXONN_ERR_INVALID_ARG
    assert L.axonn_linear_tune(5, 256, 256, 256, ALIGNED, ALIGNED, ALIGNED, None, 0, None, ctypes.byref(res)) == bad
    assert L.axonn_linear_tune(0, 0, 256, 256, ALIGNED, ALIGNED, ALIGNED, None, 0, None, ctypes.byref(res)) == bad
    assert L.axonn_linear_tune(0, 256, 256, 256, 0, ALIGNED, ALIGNED, None, 0, None, ctypes.byref(res)) == bad
    assert L.axonn_linear_tune(0, 256, 256, 256, ALIGNED, ALIGNED, ALIGNED, ALIGNED + 16, 1 << 20, None, ctypes.byref(res)) == bad
    assert L.axonn_linear_tune(0, 256, 256, 256, ALIGNED, ALIGNED, ALIGNED, None, 0, None, None) == bad


# ------------------------------------------------------------------ launch plans (host logic)
@pytest.mark.parametrize("shape", [(2048, 12288, 4096), (12288, 2048, 4096), (4096, 5120, 4096), (6144, 6144, 6144),
                                   (2048, 16384, 4096), (2048, 4096, 4096), (256, 256, 256), (100, 100, 64),
                                   (2560, 8192, 1024), (2048, 10240, 1024), (128, 65536, 512), (2048, 4608, 18432),
                                   (2048, 6144, 49152)])
@pytest.mark.parametrize("layout", ["NN", "NT", "TN"])
def test_plan_blocks_tile_the_output_and_their_variants_fit(shape, layout):
    M, N, K = shape
    parts = B.plan(M, N, K, layout)
    assert 1 <= len(parts) <= 2
    for p in parts:
        assert B.variant_name(p["variant"]) != "mfma16_edge_128x128" or (M % 128 or N % 128)
    first = parts[0]
    assert (first["row0"], first["col0"]) == (0, 0)
    if len(parts) == 1:
        assert (first["m"], first["n"]) == (M, N)
        assert first["variant"] == B.select_variant(M, N, K, layout)
    else:
        second = parts[1]
        if second["col0"]:      # cut along N
            assert first["m"] == second["m"] == M and second["row0"] == 0
            assert second["col0"] == first["n"] and first["n"] + second["n"] == N
        else:                   # cut along M
            assert first["n"] == second["n"] == N and second["col0"] == 0
            assert second["row0"] == first["m"] and first["m"] + second["m"] == M
        # operand and output blocks start on 16-byte boundaries in every layout
        assert second["row0"] % 8 == 0 and second["col0"] % 8 == 0
    for p in parts:
        assert p["variant"] > 0 or len(parts) == 1
        assert B.variant_supports(p["variant"], p["m"], p["n"], K, layout)


@pytest.mark.parametrize("shape", [(2048 + 40, 4096 + 72, 1024), (2048, 4096 + 8, 4096), (2048 + 1, 4096, 4096),
                                   (2048 + 100, 12288 + 1, 4096), (129, 129, 65536), (1000, 1000, 1024),
                                   (4096, 4100, 1000), (200, 200, 64), (127, 4096, 4096), (4096, 5, 4096),
                                   (4096 + 8, 8192 + 8, 2048)])
@pytest.mark.parametrize("layout", ["NN", "NT", "TN"])
def test_plan_of_a_ragged_output_whole_tiles_then_edge_strips(shape, layout):
    M, N, K = shape
    parts = B.plan(M, N, K, layout)
    assert 1 <= len(parts) <= B.MAX_PLAN_PARTS
    edge = B.num_variants() - 1
    # the blocks are disjoint and cover the output
    cover = np.zeros((M, N), np.uint8)
    for p in parts:
        assert p["m"] > 0 and p["n"] > 0 and p["row0"] >= 0 and p["col0"] >= 0
        assert p["row0"] + p["m"] <= M and p["col0"] + p["n"] <= N
        cover[p["row0"]:p["row0"] + p["m"], p["col0"]:p["col0"] + p["n"]] += 1
        assert B.variant_supports(p["variant"], p["m"], p["n"], K, layout)
    assert cover.min() == 1 and cover.max() == 1
    mm, nm = M - M % 128, N - N % 128
    tiled = [p for p in parts if p["variant"] != edge]
    strips = [p for p in parts if p["variant"] == edge]
    if tiled:
        # tile kernels on the whole tiles, the guarded kernel on what is left
        assert K % 64 == 0 and sum(p["m"] * p["n"] for p in tiled) == mm * nm
        assert len(strips) == (M != mm) + (N != nm)
        assert B.axonn_linear_workspace_bytes(M, N, K, layout) == B.axonn_linear_workspace_bytes(mm, nm, K, layout)
    else:
        assert len(parts) == 1


def test_ragged_plan_takes_strips_only_where_they_pay():
    # a strip is a chain of K/128 steps of about 2 us each: worth it beside a large tiled part ...
    edge = B.num_variants() - 1
    for shape in [(2049, 16384, 4096), (2048, 16392, 4096), (4096 + 8, 8192 + 8, 2048), (2048 + 104, 12288 + 8, 4096)]:
        for lay in ("NN", "NT", "TN"):
            parts = B.plan(*shape, lay)
            if lay == "TN" and shape[0] % 8:
                # the tile kernels want every row of A (stored [K, M]) on a 16-byte boundary
                assert len(parts) == 1 and parts[0]["variant"] == edge, (shape, lay, parts)
                continue
            assert len(parts) >= 2 and parts[0]["variant"] != edge and parts[-1]["variant"] == edge, (shape, lay, parts)
    # ... and not beside a small one, nor when K does not suit the tile kernels
    # ... nor when the rows of the output would start off 16-byte boundaries (N not a multiple of 8)
    for shape in [(2088, 4168, 1024), (1064, 1608, 768), (200, 200, 64), (4096, 4100, 1000), (2049, 16384, 4010),
                  (2048, 16384 + 4, 4096), (2048 + 100, 12288 + 1, 4096)]:
        for lay in ("NN", "NT", "TN"):
            parts = B.plan(*shape, lay)
            assert len(parts) == 1 and parts[0]["variant"] == edge, (shape, lay, parts)


def test_plan_cuts_one_and_a_half_rounds_and_leaves_whole_rounds_alone():
    # 384 tiles of 256x256 on 256 compute units: a block of 256 tiles, then the other 128
    parts = B.plan(2048, 12288, 4096, "NN")
    assert [(p["m"], p["n"]) for p in parts] == [(2048, 8192), (2048, 4096)]
    assert B.variant_name(parts[0]["variant"]).endswith("256x256_w8")
    # 512 tiles: two whole rounds, one launch; 128 tiles: one launch (split-K or a smaller tile)
    assert len(B.plan(2048, 16384, 4096, "NN")) == 1
    assert len(B.plan(2048, 4096, 4096, "NN")) == 1
    # the workspace a caller must bring covers the split-K block of a plan
    parts = B.plan(2048, 12288, 8192, "NT")
    assert B.variant_name(parts[1]["variant"]).endswith("sk2")
    assert B.axonn_linear_workspace_bytes(2048, 12288, 8192, "NT") == 4096 + 128 * 256 * 256 * 4


def test_plan_rejects_bad_arguments():
    import ctypes
    L = B.lib()
    parts = (B.PlanPart * 2)()
    assert L.axonn_linear_plan(0, 128, 128, 0, parts) == B.AXONN_ERR_INVALID_ARG
    assert L.axonn_linear_plan(128, 128, 128, 3, parts) == B.AXONN_ERR_INVALID_ARG
    assert L.axonn_linear_plan(128, 128, 128, 0, ctypes.cast(None, ctypes.POINTER(B.PlanPart))) == B.AXONN_ERR_INVALID_ARG


def test_amd_smi_text_is_parsed():
    from paper_2502_08145_amd.sweeps import parse_smi
    text = """GPU: 0
    POWER:
        SOCKET_POWER: 1398 W
        GFX_VOLTAGE: N/A
    CLOCK:
        GFX_0:
            CLK: 1915 MHz
            MIN_CLK: 500 MHz
            MAX_CLK: 2400 MHz
        GFX_1:
            CLK: 1865 MHz
            MIN_CLK: 500 MHz
        MEM_0:
            CLK: 2000 MHz
"""
    assert parse_smi(text) == (1398, [1915, 1865])
    assert parse_smi("no such fields") == (None, [])


def test_source_hash_ignores_comments_and_blank_space(tmp_path, monkeypatch):
    """The hash that ties stored counter readings to a build changes with the code, not with its comments."""
    from paper_2502_08145_amd import build
    csrc = tmp_path / "pkg" / "csrc"
    inc = tmp_path / "include"
    csrc.mkdir(parents=True)
    inc.mkdir()
    (inc / "axonn_linear.h").write_text("int f(void);\n")
    monkeypatch.setattr(build, "CSRC", str(csrc))
    monkeypatch.setattr(build, "HERE", str(tmp_path / "pkg"))
    (csrc / "k.hpp").write_text("// a comment\nint   x = 1;   /* block\n comment */\n\nint y = 2;\n")
    first = build.source_id()
    (csrc / "k.hpp").write_text("int x = 1;\nint y = 2;  // another comment\n")
    assert build.source_id() == first
    (csrc / "k.hpp").write_text("int x = 1;\nint y = 3;\n")
    assert build.source_id() != first
    (csrc / "notes.orig").write_text("not a source file")
    (csrc / "k.hpp").write_text("int x = 1;\nint y = 2;\n")
    assert build.source_id() == first


def test_planner_choices_that_the_design_notes_describe():
    """Host-only: the selection model on a few shapes whose plans are stated in the design notes."""
    name = lambda M, N, K, lay: B.plan_name(M, N, K, lay)
    # narrow outputs over a long K: half tiles in three K ranges (64-k kernel for NT, 32-k ring for NN)
    assert name(2048, 1152, 36864, "NT") == "mfma16k64_256x128_sk3"
    assert name(2048, 1152, 36864, "NN") == "mfma16_256x128_sk3"
    # 128 large tiles at K = 4096: half tiles with 64-k stages for NT, the ring's half tiles for NN
    assert name(2048, 4096, 4096, "NT") == "mfma16k64_256x128"
    assert name(2048, 4096, 4096, "NN") == "mfma16_128x256"
    # the resident kernel: TN from three rounds on up to K = 8192, NN at K <= 2048; not at long K
    assert name(4096, 16384, 2048, "TN") == "mfma16k64p_256x256_w8"
    assert name(4096, 16384, 2048, "NN") == "mfma16k64p_256x256_w8"
    assert name(16384, 16384, 16384, "TN") == "mfma16k64_256x256_w8"
    assert name(4096, 16384, 2048, "NT") == "mfma16k64_256x256_w8"
    # NT at long K stays on the 64-k kernel (its A panel is triple-buffered), also when split
    assert name(8192, 8192, 32768, "NT") == "mfma16k64_256x256_w8"
    assert name(2048, 2048, 65536, "NT").startswith("mfma16k64_256x256_w8_sk")
    # one and a half rounds of large tiles: two launches
    assert "+" in name(2048, 12288, 4096, "NN")
