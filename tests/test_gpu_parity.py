"""GPU parity: every result of the HIP library is compared with the CPU oracle on the same
seeded inputs, through the C ABI (binding.py only marshals arguments).

Tolerance (written here as in tests/gpu_util.py): normwise relative error <= 1e-2 and
elementwise error <= 2e-2 * max|ref|; integer-valued inputs must match RNE_bf16(ref) bit for
bit, because every partial sum is then an integer below 2^24 and exact in fp32 under any
summation order.
"""
import numpy as np
import pytest
import torch

from paper_2502_08145_amd import binding as B
from paper_2502_08145_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

LAYOUTS = ["NN", "NT", "TN"]
OPS = ["fwd", "bwd_data", "bwd_weight"]


def store(a_mk, b_kn, layout):
    if layout == "NN":
        return a_mk, b_kn
    if layout == "NT":
        return a_mk, synth.transpose_bits(b_kn)
    return synth.transpose_bits(a_mk), b_kn


def run_gpu(op, M, N, K, layout, A_bits, B_bits, variant=-1, stream=None, poison=True):
    a, b = U.to_device(A_bits), U.to_device(B_bits)
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    if poison:
        c.view(torch.int16).fill_(0x7FC0)  # bf16 NaN pattern: unwritten output shows up
    B.force_variant(variant)
    try:
        B.OPS[op](M, N, K, layout, a, b, c, 1, stream)
    finally:
        B.force_variant(-1)
    torch.cuda.synchronize()
    return U.to_host_bits(c)


def run_gpu_guard_rows(op, M, N, K, layout, A_bits, B_bits, variant=-1):
    """run_gpu with two more rows behind the output, which must come back untouched."""
    a, b = U.to_device(A_bits), U.to_device(B_bits)
    buf = torch.empty((M + 2, N), dtype=torch.bfloat16, device="cuda")
    buf.view(torch.int16).fill_(0x7FC0)
    B.force_variant(variant)
    try:
        B.OPS[op](M, N, K, layout, a, b, buf[:M], 1, None)
    finally:
        B.force_variant(-1)
    torch.cuda.synchronize()
    host = U.to_host_bits(buf)
    assert (host[M:] == 0x7FC0).all(), "rows behind the output were written"
    return host[:M]


def tile_variants(layout=None):
    """All MFMA tile variants that have a kernel for `layout` (the half tiles with 64-k stages exist for NT
    only); the last variant is the guarded one."""
    vs = list(range(1, edge_variant()))
    if layout is None:
        return vs
    return [v for v in vs if B.variant_supports(v, 256, 256, 64 * 840, layout)]   # 840 K-steps: any number of K ranges up to 8


def edge_variant():
    v = B.num_variants() - 1
    assert B.variant_name(v) == "mfma16_edge_128x128"
    return v


def splits_of(v):
    """K ranges per tile of a variant (split-K variants are named ..._sk<ranges>)."""
    tail = B.variant_name(v).rsplit("_", 1)[-1]
    return int(tail[2:]) if tail.startswith("sk") else 1


def kstep_of(v):
    """K granularity of a variant: every tile kernel consumes K 64 at a time."""
    return 64


def usable(v, M, N, K, layout):
    """Every plain tile variant must take the test shape; a split-K one may decline it."""
    ok = B.variant_supports(v, M, N, K, layout)
    assert ok or splits_of(v) > 1, (B.variant_name(v), M, N, K, layout)
    return ok


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-test] {request.node.name}", flush=True)
    yield


@pytest.fixture(autouse=True)
def _workspace():
    """The library allocates nothing: every test runs with a torch-owned split-K scratch area of the
    largest size any product needs, registered afresh (tests that register their own restore this)."""
    U.shared_workspace()
    yield


# ------------------------------------------------------------------ ragged shapes, guarded kernel
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (17, 1, 33), (1, 64, 1), (37, 53, 71), (130, 257, 65)])
def test_ragged_shapes_any_size(oracle_mod, layout, shape):
    M, N, K = shape
    a = synth.normal_bf16(1000 + M, (M, K))
    b = synth.normal_bf16(2000 + N, (K, N), 0.02)
    A, Bm = store(a, b, layout)
    ref = oracle_mod.gemm(M, N, K, layout, A, Bm)
    assert B.select_variant(M, N, K, layout) == edge_variant()
    for op in OPS:
        got = run_gpu(op, M, N, K, layout, A, Bm)
        U.assert_close(got, ref, f"{op} {layout} {shape}")
    got = run_gpu("fwd", M, N, K, layout, A, Bm, variant=0)
    U.assert_close(got, ref, f"naive {layout} {shape}")


# ------------------------------------------------------------------ the guarded MFMA kernel
@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", [(300, 270, 100), (257, 129, 200), (128, 128, 32), (129, 127, 31), (640, 384, 352),
                                   (5, 1000, 515), (1000, 5, 1027), (264, 392, 8)])
def test_guarded_mfma_kernel_bit_exact_on_integers(oracle_mod, layout, shape):
    # several tiles, ragged tails in all three directions, leading dimensions that leave rows at odd
    # addresses (no vector loads), K shorter than a K-step; small integers: the sum is exact in
    # fp32 and the output must equal the rounded oracle bit for bit
    M, N, K = shape
    a = synth.integer_bf16(500 + M, (M, K), -4, 4)
    b = synth.integer_bf16(600 + N, (K, N), -4, 4)
    A, Bm = store(a, b, layout)
    want = U.f64_to_bf16_bits_rne(oracle_mod.gemm(M, N, K, layout, A, Bm))
    got = run_gpu_guard_rows("fwd", M, N, K, layout, A, Bm, variant=edge_variant())
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"{layout} {shape}: {len(bad)} mismatches, first at {bad[0]}"


@pytest.mark.parametrize("layout", LAYOUTS)
def test_guarded_mfma_kernel_against_oracle_normal_data(oracle_mod, layout):
    for M, N, K in [(768, 768, 416), (391, 1003, 777)]:
        a = synth.normal_bf16(71 + M, (M, K))
        b = synth.normal_bf16(72 + N, (K, N), 0.02)
        A, Bm = store(a, b, layout)
        ref = oracle_mod.gemm(M, N, K, layout, A, Bm)
        got = run_gpu("fwd", M, N, K, layout, A, Bm, variant=edge_variant())
        nw, ew = U.assert_close(got, ref, f"edge {layout} {(M, N, K)}")
        assert nw < 4e-3, nw


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", [(1024 + 40, 1536 + 72, 768), (1152, 1024 + 8, 1024), (1024 + 1, 1280, 1024)])
def test_ragged_output_of_several_tiles_every_element(oracle_mod, layout, shape):
    # every element, bit for bit on integer data, through all three entry points, and nothing
    # written behind the output
    M, N, K = shape
    a = synth.integer_bf16(700 + M, (M, K), -4, 4)
    b = synth.integer_bf16(800 + N, (K, N), -4, 4)
    A, Bm = store(a, b, layout)
    want = U.f64_to_bf16_bits_rne(oracle_mod.gemm(M, N, K, layout, A, Bm))
    for op in OPS:
        got = run_gpu_guard_rows(op, M, N, K, layout, A, Bm)
        bad = np.argwhere(got != want)
        assert bad.size == 0, f"{op} {layout} {shape}: {len(bad)} mismatches, first at {bad[0]}"


@pytest.mark.parametrize("shape", [(4096 + 8, 8192 + 8, 2048), (2048 + 1, 8192, 2048), (4096, 8192 + 104, 2048)])
def test_ragged_output_as_tiles_plus_edge_strips_sampled(oracle_mod, shape):
    """A large ragged output: whole tiles by the tile kernels, the last columns and the last rows by
    the guarded kernel as launches of their own.  Integer data; the strips in full, the tiled part
    on sampled rows, columns and one element per 128 x 128 block, bit for bit."""
    M, N, K = shape
    mm, nm = M - M % 128, N - N % 128
    a = synth.integer_bf16(900 + M, (M, K), -4, 4)
    b = synth.integer_bf16(901 + N, (K, N), -4, 4)
    ii, jj = _sample_positions(M, N, seed=M + N)
    si, sj = np.nonzero(np.add.outer(np.arange(M) >= mm, np.arange(N) >= nm))   # the strips, every element
    ii, jj = np.concatenate([ii, si]), np.concatenate([jj, sj])
    want = U.f64_to_bf16_bits_rne(oracle_mod.gemm_at(M, N, K, "NN", a, b, ii, jj))
    for layout in LAYOUTS:
        parts = B.plan(M, N, K, layout)
        if layout == "TN" and M % 8:
            assert len(parts) == 1 and parts[0]["variant"] == edge_variant()   # rows of A off 16-byte boundaries
        else:
            assert len(parts) >= 1 + (M != mm) + (N != nm) and parts[0]["variant"] != edge_variant(), parts
            assert [p["variant"] for p in parts].count(edge_variant()) == (M != mm) + (N != nm)
        A, Bm = store(a, b, layout)
        got = run_gpu_guard_rows("fwd", M, N, K, layout, A, Bm)
        assert np.isfinite(U.bits_to_f64(got)).all(), f"{shape} {layout}: unwritten or non-finite output"
        bad = np.nonzero(got[ii, jj] != want)[0]
        assert bad.size == 0, f"{layout} {shape}: {len(bad)} mismatches, first at {(ii[bad[0]], jj[bad[0]])}"


def test_k_zero_gives_zero_and_empty_outputs_are_ok():
    c = torch.full((8, 16), 3.0, dtype=torch.bfloat16, device="cuda")
    a = torch.empty((8, 0), dtype=torch.bfloat16, device="cuda")
    b = torch.empty((0, 16), dtype=torch.bfloat16, device="cuda")
    B.axonn_linear_fwd(8, 16, 0, "NN", a, b, c)
    torch.cuda.synchronize()
    assert np.array_equal(U.to_host_bits(c), np.zeros((8, 16), np.uint16))
    assert B.axonn_linear_fwd(0, 16, 8, "NN", 0, 0, 0, check=False) == B.AXONN_OK


# ------------------------------------------------------------------ every tile kernel, several tiles
@pytest.mark.parametrize("layout", LAYOUTS)
def test_every_tile_variant_against_oracle(oracle_mod, layout):
    # 3 x 3 tiles of 256 (6 x 6 of 128), 7 K-steps of 64 per workgroup: multi-tile, the LDS ring
    # wraps twice; split-K variants get 7 steps per K range (9 tiles x splits workgroups is not a
    # multiple of 8: the plain workgroup -> tile mapping)
    M, N = 768, 768
    for splits in range(1, 9):
        K = 448 * splits
        a = synth.normal_bf16(31 + splits, (M, K))
        b = synth.normal_bf16(32 + splits, (K, N), 0.02)
        A, Bm = store(a, b, layout)
        ref = oracle_mod.gemm(M, N, K, layout, A, Bm)
        ran = 0
        for v in tile_variants(layout):
            if splits_of(v) != splits:
                continue
            assert B.variant_supports(v, M, N, K, layout)
            got = run_gpu("fwd", M, N, K, layout, A, Bm, variant=v)
            nw, ew = U.assert_close(got, ref, f"{B.variant_name(v)} {layout}")
            # a correct kernel sits near the bf16 rounding floor (2^-9 rms), far inside the bound
            assert nw < 4e-3, (B.variant_name(v), nw)
            ran += 1
        # one range: 7 kernels for every mode and the two half tiles with 64-k stages for NT; split: the large
        # tile on both kernels (and 128 x 128 in two and four ranges); in two and three ranges also the ring's
        # half tiles and, for NT, the half tiles with 64-k stages
        expect = (9 if layout == "NT" else 7) if splits == 1 else {2: 3, 4: 3}.get(splits, 2) + ((4 if layout == "NT" else 2) if splits <= 3 else 0)
        assert ran == expect, (splits, ran)
    assert B.axonn_linear_split_k_timeouts() == 0


@pytest.mark.parametrize("layout", LAYOUTS)
def test_split_k_xcd_mapping_and_repeated_launches(oracle_mod, layout):
    # 2 x 4 tiles of 256: the workgroup count is a multiple of 8 * splits, the mapping that keeps the
    # workgroups of one tile on one XCD.  Three launches in a row reuse the same scratch slots with
    # a new epoch each; integer data makes the comparison exact.  K = 384 per range.
    M, N = 512, 1024
    ran = 0
    for splits in range(2, 9):
        K = 384 * splits
        a = synth.integer_bf16(91 + splits, (M, K), -4, 4)
        b = synth.integer_bf16(92 + splits, (K, N), -4, 4)
        A, Bm = store(a, b, layout)
        want = U.f64_to_bf16_bits_rne(oracle_mod.gemm(M, N, K, layout, A, Bm))
        for v in tile_variants(layout):
            if splits_of(v) != splits:
                continue
            assert B.variant_supports(v, M, N, K, layout)
            for rep in range(3):
                got = run_gpu("bwd_data", M, N, K, layout, A, Bm, variant=v)
                assert np.array_equal(got, want), f"{B.variant_name(v)} {layout} launch {rep}"
            ran += 1
    assert ran == (24 if layout == "NT" else 20)
    assert B.axonn_linear_split_k_timeouts() == 0


@pytest.mark.parametrize("shape", [(512, 512, 32768), (256, 512, 32768), (768, 256, 32768)])
@pytest.mark.parametrize("layout", LAYOUTS)
def test_split_k_long_k_one_range_per_xcd_pair(oracle_mod, layout, shape):
    # From K = 32768 on, the 256x256 kernels with four K ranges give each pair of XCDs one range
    # (workgroup count a multiple of 8: 4 and 2 tiles; 3 tiles fall back to the plain order).
    # Integer data: exact under any order of the partial sums (|sum| <= 16 K < 2^24).
    M, N, K = shape
    a = synth.integer_bf16(95, (M, K), -4, 4)
    b = synth.integer_bf16(96, (K, N), -4, 4)
    A, Bm = store(a, b, layout)
    want = U.f64_to_bf16_bits_rne(oracle_mod.gemm(M, N, K, layout, A, Bm))
    ran = 0
    for v in tile_variants(layout):
        if splits_of(v) != 4 or "256x256" not in B.variant_name(v):
            continue
        assert B.variant_supports(v, M, N, K, layout)
        for rep in range(2):
            got = run_gpu("fwd", M, N, K, layout, A, Bm, variant=v)
            assert np.array_equal(got, want), f"{B.variant_name(v)} {layout} launch {rep}"
        ran += 1
    assert ran == 2
    assert B.axonn_linear_split_k_timeouts() == 0


@pytest.mark.parametrize("layout", LAYOUTS)
def test_shortest_k_and_single_tile(oracle_mod, layout):
    # the shortest K each tile kernel takes (its prologue fills the whole LDS ring, the main loop
    # never runs), and one step more
    M = N = 256
    for v in tile_variants(layout):
        kmin = next(k for k in range(64, 4096, 64) if B.variant_supports(v, M, N, k, layout))
        assert not B.variant_supports(v, M, N, kmin - 64, layout) and not B.variant_supports(v, M, N, kmin + 32, layout)
        for K in (kmin, kmin + kstep_of(v) * splits_of(v)):
            a = synth.normal_bf16(41 + K, (M, K))
            b = synth.normal_bf16(42 + K, (K, N))
            A, Bm = store(a, b, layout)
            ref = oracle_mod.gemm(M, N, K, layout, A, Bm)
            got = run_gpu("bwd_data", M, N, K, layout, A, Bm, variant=v)
            U.assert_close(got, ref, f"{B.variant_name(v)} {layout} K={K}")


def test_caller_owned_workspace(oracle_mod):
    # the same split-K problem through a registered buffer that is large enough, with one that is too
    # small (automatic choice then avoids split-K, a forced split-K variant is refused) and with none
    M, N, K, layout = 512, 1024, 1792, "NT"
    a = synth.integer_bf16(93, (M, K), -4, 4)
    b = synth.integer_bf16(94, (K, N), -4, 4)
    A, Bm = store(a, b, layout)
    want = U.f64_to_bf16_bits_rne(oracle_mod.gemm(M, N, K, layout, A, Bm))
    sk2 = next(v for v in tile_variants() if B.variant_name(v) == "mfma16_256x256_w8_sk2")
    need = 4096 + 8 * 256 * 256 * 4
    M2, N2, K2 = 1024, 1024, 4096        # a split-K-worthy shape for the automatic choice
    a2 = synth.integer_bf16(95, (M2, K2), -4, 4)
    b2 = synth.integer_bf16(96, (K2, N2), -4, 4)
    A2, B2 = store(a2, b2, layout)
    want2 = U.f64_to_bf16_bits_rne(oracle_mod.gemm(M2, N2, K2, layout, A2, B2))
    assert "_sk" in B.plan_name(M2, N2, K2, layout)
    try:
        big = torch.full((need + 4096,), 0x55, dtype=torch.uint8, device="cuda")     # dirty on purpose
        B.axonn_linear_set_workspace(big)
        for rep in range(2):
            assert np.array_equal(run_gpu("fwd", M, N, K, layout, A, Bm, variant=sk2), want)
        # every flag a writer raised has been taken down again by its reader (a launch replayed from
        # a captured graph carries the same epoch again and must not find it standing)
        flags = big[:4096].view(torch.int32).cpu().numpy()
        assert not flags[:1023].any() and flags[1023] == 0, "split-K flags left standing, or a time-out"
        # ... also by the other kernel families
        for name in ("mfma16k64_256x256_w8_sk2", "mfma16_128x128_sk2"):
            v16 = [B.variant_name(v) for v in range(B.num_variants())].index(name)
            assert np.array_equal(run_gpu("fwd", M, N, K, layout, A, Bm, variant=v16), want), name
            assert not big[:4096].view(torch.int32).cpu().numpy().any(), name
        small = torch.zeros((4096 + 3 * 256 * 256 * 4,), dtype=torch.uint8, device="cuda")
        B.axonn_linear_set_workspace(small)
        B.force_variant(sk2)
        try:
            c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
            rc = B.axonn_linear_fwd(M, N, K, layout, U.to_device(A), U.to_device(Bm), c, check=False)
            assert rc == B.AXONN_ERR_WORKSPACE
        finally:
            B.force_variant(-1)
        # automatic selection for a split-K-worthy shape still gives the right answer, without split-K
        assert B.axonn_linear_workspace_bytes(M2, N2, K2, layout) > small.numel()
        assert "_sk" not in B.plan_name(M2, N2, K2, layout, now=True)
        assert np.array_equal(run_gpu("fwd", M2, N2, K2, layout, A2, B2), want2)
        # no area registered at all: the library allocates none of its own
        torch.cuda.synchronize()
        B.axonn_linear_set_workspace(None)
        big.fill_(0x55)
        torch.cuda.synchronize()
        assert "_sk" not in B.plan_name(M2, N2, K2, layout, now=True)
        assert np.array_equal(run_gpu("fwd", M2, N2, K2, layout, A2, B2), want2)
        B.force_variant(sk2)
        try:
            c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
            rc = B.axonn_linear_fwd(M, N, K, layout, U.to_device(A), U.to_device(Bm), c, check=False)
            assert rc == B.AXONN_ERR_WORKSPACE
        finally:
            B.force_variant(-1)
        assert B.axonn_linear_split_k_timeouts() == 0
        assert (big == 0x55).all(), "an unregistered buffer was written"
        # exactly the advertised size is accepted, for a plan of small tiles too
        for shape in ((M2, N2, K2), (128, 128, 8192)):
            nb = B.axonn_linear_workspace_bytes(*shape, layout)
            assert nb >= 4096 + 256 * 256 * 4
            exact = torch.zeros((nb,), dtype=torch.uint8, device="cuda")
            B.axonn_linear_set_workspace(exact)
            assert B.plan_name(*shape, layout, now=True) == B.plan_name(*shape, layout)
        assert np.array_equal(run_gpu("fwd", M2, N2, K2, layout, A2, B2), want2)
    finally:
        U.shared_workspace()
    assert "_sk" in B.plan_name(M2, N2, K2, layout, now=True)
    assert np.array_equal(run_gpu("fwd", M, N, K, layout, A, Bm, variant=sk2), want)
    assert B.axonn_linear_split_k_timeouts() == 0


# ------------------------------------------------------------------ exact integers: bit for bit
@pytest.mark.parametrize("layout", LAYOUTS)
def test_integer_inputs_are_bit_exact(oracle_mod, layout):
    M, N, K = 512, 768, 1536   # rectangular, 2 x 3 tiles of 256, 48 K-steps (12 per range when split in 4)
    a = synth.integer_bf16(51, (M, K), -4, 4)
    b = synth.integer_bf16(52, (K, N), -4, 4)
    A, Bm = store(a, b, layout)
    ref = oracle_mod.gemm(M, N, K, layout, A, Bm)
    want = U.f64_to_bf16_bits_rne(ref)
    for v in [0] + tile_variants(layout):
        if splits_of(v) in (5, 7):     # K is not a multiple of 5 or 7 K ranges of whole K-steps
            continue
        assert B.variant_supports(v, M, N, K, layout)
        got = run_gpu("bwd_weight", M, N, K, layout, A, Bm, variant=v)
        bad = np.argwhere(got != want)
        assert bad.size == 0, f"{B.variant_name(v)} {layout}: {len(bad)} mismatches, first at {bad[0]}"


@pytest.mark.parametrize("layout", LAYOUTS)
def test_position_coded_operands_catch_any_index_slip(oracle_mod, layout):
    # A is one-hot per row with a row-dependent column, B holds a distinct exact value per
    # (k, j): C[i, j] = B[sel(i), j], exact in bf16, so any swapped row/column/k shows up.
    M, N, K = 512, 512, 256
    sel = (np.arange(M) * 37 + 11) % K
    a = np.zeros((M, K), np.float32)
    a[np.arange(M), sel] = 1.0
    kk, jj = np.meshgrid(np.arange(K), np.arange(N), indexing="ij")
    b = ((kk % 16) * 16 + (jj % 16) - 128).astype(np.float32) * np.where((kk // 16 + jj // 16) % 2 == 0, 1.0, 0.5)
    a_bits, b_bits = synth.f32_to_bf16_bits(a).reshape(M, K), synth.f32_to_bf16_bits(b).reshape(K, N)
    assert np.array_equal(synth.bf16_bits_to_f32(b_bits).reshape(K, N), b)
    A, Bm = store(a_bits, b_bits, layout)
    ref = oracle_mod.gemm(M, N, K, layout, A, Bm)
    assert np.array_equal(ref, b[sel].astype(np.float64))
    for v in [0] + tile_variants(layout):
        if not usable(v, M, N, K, layout):
            continue
        got = run_gpu("fwd", M, N, K, layout, A, Bm, variant=v)
        assert np.array_equal(U.bits_to_f64(got), ref), f"{B.variant_name(v)} {layout}"


# ------------------------------------------------------------------ config 1 in full: tiny GPT MLP
def test_tiny_mlp_all_ops_all_layouts(oracle_mod):
    tokens, h, ff = 1024, 512, 2048
    for tag, (d_in, d_out), seed in (("fc1", (h, ff), 100), ("fc2", (ff, h), 200)):
        t = synth.fc_layer_tensors(tokens, d_in, d_out, synth.BASE_SEED + seed)
        for g in synth.fc_layer_gemms(tokens, d_in, d_out, tag):
            ref = None
            for layout in LAYOUTS:
                A, Bm = synth.operands_for(g["op"], layout, t)
                if ref is None:   # all three modes of one GEMM have the same reference result
                    ref = oracle_mod.gemm(g["M"], g["N"], g["K"], layout, A, Bm)
                got = run_gpu(g["op"], g["M"], g["N"], g["K"], layout, A, Bm)
                U.assert_close(got, ref, f"{g['name']} {layout}")


# ------------------------------------------------------------------ determinism, streams, errors
@pytest.mark.parametrize("shape,kind", [((1024, 512, 1024), "mfma"), ((2048, 4096, 16384), "_sk"),
                                        ((1000, 520, 1031), "mfma16_edge"), ((2049, 8192, 2048), "+mfma16_edge")])
def test_same_inputs_same_bits_and_side_stream(oracle_mod, shape, kind):
    # a plain tile kernel, split-K (fixed reduction order), the guarded kernel, tiles plus an edge strip
    M, N, K = shape
    assert kind in B.plan_name(M, N, K, "NN")
    a = synth.normal_bf16(61, (M, K))
    b = synth.normal_bf16(62, (K, N))
    first = run_gpu("fwd", M, N, K, "NN", a, b)
    for _ in range(3):
        assert np.array_equal(run_gpu("fwd", M, N, K, "NN", a, b), first)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        other = run_gpu("fwd", M, N, K, "NN", a, b, stream=s)
    assert np.array_equal(other, first)


@pytest.mark.parametrize("variant,shape", [("mfma16_256x256_w8_sk2", (768, 768, 1792)), ("mfma16_128x128_sk4", (512, 384, 2048)),
                                           ("mfma16k64_256x256_w8_sk3", (512, 768, 1536)), (None, (768, 512, 448))])
def test_calls_captured_in_a_hip_graph_replay_correctly(variant, shape):
    """A captured split-K launch carries the epoch of its capture into every replay: the flags it
    raises must be down again when the next replay starts.  Replays alternate with eager work and
    synchronisations, the inputs change between them, and every replay must give the bits of an
    eager call on the same inputs."""
    M, N, K = shape
    names = [B.variant_name(v) for v in range(B.num_variants())]
    v = names.index(variant) if variant else -1
    assert v < 0 or B.variant_supports(v, M, N, K, "NT")
    gen = torch.Generator(device="cuda").manual_seed(77)
    a = torch.randn((M, K), generator=gen, device="cuda").to(torch.bfloat16)
    b = torch.randn((N, K), generator=gen, device="cuda").to(torch.bfloat16)
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    c_eager = torch.empty_like(c)
    B.force_variant(v)
    try:
        B.axonn_linear_bwd_data(M, N, K, "NT", a, b, c_eager)      # also raises the LDS limits before the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            B.axonn_linear_bwd_data(M, N, K, "NT", a, b, c, 1, torch.cuda.current_stream())
        for rep in range(5):
            a.copy_(torch.randn((M, K), generator=gen, device="cuda").to(torch.bfloat16))
            b.copy_(torch.randn((N, K), generator=gen, device="cuda").to(torch.bfloat16))
            c.view(torch.int16).fill_(0x7FC0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            B.axonn_linear_bwd_data(M, N, K, "NT", a, b, c_eager)
            torch.cuda.synchronize()
            assert torch.equal(c.view(torch.int16), c_eager.view(torch.int16)), f"replay {rep} differs from the eager call"
    finally:
        B.force_variant(-1)
    assert B.axonn_linear_split_k_timeouts() == 0


def test_forced_variant_that_cannot_run_is_refused():
    a = torch.zeros((100, 64), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((64, 100), dtype=torch.bfloat16, device="cuda")
    c = torch.zeros((100, 100), dtype=torch.bfloat16, device="cuda")
    B.force_variant(1)
    try:
        assert B.axonn_linear_fwd(100, 100, 64, "NN", a, b, c, check=False) == B.AXONN_ERR_UNSUPPORTED
    finally:
        B.force_variant(-1)
    assert B.axonn_linear_fwd(100, 100, 64, "NN", a, b, c, check=False) == B.AXONN_OK
    torch.cuda.synchronize()


# ------------------------------------------------------------------ full benchmark sizes, sampled
def _sample_positions(M, N, seed, n_rows=4, n_cols=4, block=128):
    rng = np.random.default_rng(seed)
    ii, jj = [], []
    for r in rng.choice(M, size=min(n_rows, M), replace=False):          # full rows
        ii.append(np.full(N, r)); jj.append(np.arange(N))
    for c in rng.choice(N, size=min(n_cols, N), replace=False):          # full columns
        ii.append(np.arange(M)); jj.append(np.full(M, c))
    bi, bj = np.meshgrid(np.arange(0, M, block), np.arange(0, N, block), indexing="ij")   # one per block
    ii.append((bi + rng.integers(0, block, bi.shape)).ravel().clip(max=M - 1))
    jj.append((bj + rng.integers(0, block, bj.shape)).ravel().clip(max=N - 1))
    return np.concatenate(ii).astype(np.int64), np.concatenate(jj).astype(np.int64)


FULL_SIZE = [
    # (name, tokens, d_in, d_out): every layer of the benchmark workloads above the tiny one
    ("gpt5b.qkv", 2048, 4096, 12288),
    ("gpt5b.attn_out", 2048, 4096, 4096),
    ("gpt5b.fc1", 2048, 4096, 16384),
    ("gpt5b.fc2", 2048, 16384, 4096),
    ("gpt80b_shard.fc1", 4096, 2048, 16384),
    ("gpt80b_shard.fc2", 4096, 16384, 2048),
    ("gpt320b_skinny.fc1", 2048, 2048, 8192),
    ("gpt320b_skinny.fc2", 2048, 8192, 2048),
]


@pytest.mark.parametrize("name,tokens,d_in,d_out", FULL_SIZE)
def test_full_size_layers_every_element(oracle_mod, name, tokens, d_in, d_out):
    """Benchmark-size GEMMs in the launch configuration bench.py times (automatic plan, split-K
    scratch registered): forward, backward-data and backward-weight of the layer, each in all three
    modes, the WHOLE output against the whole oracle product."""
    t = synth.fc_layer_tensors(tokens, d_in, d_out, synth.BASE_SEED + 300)
    for g in synth.fc_layer_gemms(tokens, d_in, d_out, name):
        M, N, K = g["M"], g["N"], g["K"]
        A, Bm = synth.operands_for(g["op"], g["layout"], t)
        print(f"  {g['name']} {M}x{N}x{K}: oracle ...", flush=True)
        ref = oracle_mod.gemm(M, N, K, g["layout"], A, Bm)
        for layout in LAYOUTS:   # all three modes of one GEMM have the same reference result
            A, Bm = synth.operands_for(g["op"], layout, t)
            assert B.plan_name(M, N, K, layout, now=True) == B.plan_name(M, N, K, layout)
            got = run_gpu(g["op"], M, N, K, layout, A, Bm)
            nw, ew = U.assert_close(got, ref, f"{g['name']} {layout}")
            assert nw < 4e-3, (g["name"], layout, nw)   # the bf16 rounding floor is 2^-9 rms
        del ref


@pytest.mark.parametrize("name,tokens,d_in,d_out", FULL_SIZE)
def test_full_size_layers_integer_data_bit_for_bit(oracle_mod, name, tokens, d_in, d_out):
    """The same shapes on integer-valued operands in their natural modes (the launches bench.py times):
    every partial sum is an integer below 2^24, exact in fp32 whatever the order, so sampled rows,
    columns and one element per 128 x 128 block must equal the rounded oracle value bit for bit."""
    t = dict(X=synth.integer_bf16(synth.BASE_SEED + 310, (tokens, d_in), -4, 4),
             W=synth.integer_bf16(synth.BASE_SEED + 311, (d_in, d_out), -4, 4),
             dY=synth.integer_bf16(synth.BASE_SEED + 312, (tokens, d_out), -4, 4))
    for g in synth.fc_layer_gemms(tokens, d_in, d_out, name):
        M, N, K = g["M"], g["N"], g["K"]
        ii, jj = _sample_positions(M, N, seed=M + 3 * N)
        A, Bm = synth.operands_for(g["op"], g["layout"], t)
        want = U.f64_to_bf16_bits_rne(oracle_mod.gemm_at(M, N, K, g["layout"], A, Bm, ii, jj))
        got = run_gpu(g["op"], M, N, K, g["layout"], A, Bm)
        assert np.isfinite(U.bits_to_f64(got)).all(), f"{g['name']}: unwritten or non-finite output"
        bad = np.nonzero(got[ii, jj] != want)[0]
        assert bad.size == 0, f"{g['name']}: {len(bad)} mismatches, first at {(ii[bad[0]], jj[bad[0]])}"


@pytest.mark.parametrize("n", [1024, 2048, 4096, 8192])
def test_square_layout_sweep_every_element(oracle_mod, n):
    """Square products of the layout sweep and of the empirical-peak curve (the paper's single-GPU GEMM
    benchmark, Sec. V-C), whole output, all three modes."""
    a = synth.normal_bf16(synth.BASE_SEED + 500, (n, n))
    b = synth.normal_bf16(synth.BASE_SEED + 501, (n, n))
    ref = oracle_mod.gemm(n, n, n, "NN", a, b)
    for layout in LAYOUTS:
        A, Bm = store(a, b, layout)
        got = run_gpu("fwd", n, n, n, layout, A, Bm)
        nw, ew = U.assert_close(got, ref, f"square {n} {layout}")
        assert nw < 4e-3, (n, layout, nw)


def test_square_16384_sampled(oracle_mod):
    n = 16384
    a = synth.normal_bf16(synth.BASE_SEED + 500, (n, n))
    b = synth.normal_bf16(synth.BASE_SEED + 501, (n, n))
    ii, jj = _sample_positions(n, n, seed=n, n_rows=2, n_cols=2)
    ref = oracle_mod.gemm_at(n, n, n, "NN", a, b, ii, jj)
    for layout in LAYOUTS:
        A, Bm = store(a, b, layout)
        got = run_gpu("fwd", n, n, n, layout, A, Bm)
        assert np.isfinite(U.bits_to_f64(got)).all()
        U.assert_close(got[ii, jj], ref, f"square {n} {layout}")


def _periodic_rows(seed, rows, cols, period, sigma=1.0):
    """[rows, cols] whose rows repeat a seeded block of `period` rows (fast to make at sizes where
    drawing every element on the host would take minutes)."""
    block = synth.normal_bf16(seed, (period, cols), sigma)
    reps = -(-rows // period)
    return np.ascontiguousarray(np.tile(block, (reps, 1))[:rows])


@pytest.mark.parametrize("n", [32768, 65536])
def test_largest_squares_of_the_peak_curve_sampled(oracle_mod, n):
    """The top of the empirical-peak curve (Sec. V-C): operands of 2 and 8.6 GB, where per-lane 32-bit
    address offsets would wrap (at n = 65536 every MN-contiguous panel is above 4 GiB).  Both operands
    repeat a seeded block of 5000 rows; 5000 divides neither 32768 rows (where a 4 GiB byte offset
    wraps at n = 65536) nor any power of two, so an address that wraps lands on other data.  Outputs
    are compared on sampled rows, columns and one element per 1024 x 1024 block, all three modes; the
    other modes' operands are transposed on the device by torch (plumbing: bits moved)."""
    a = _periodic_rows(synth.BASE_SEED + 510, n, n, 5000)
    b = _periodic_rows(synth.BASE_SEED + 511, n, n, 5000)
    ii, jj = _sample_positions(n, n, seed=n, n_rows=2, n_cols=2, block=1024)
    print(f"  oracle at {len(ii)} positions ...", flush=True)
    ref = oracle_mod.gemm_at(n, n, n, "NN", a, b, ii, jj)
    a_d, b_d = U.to_device(a), U.to_device(b)
    del a, b
    c = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
    ti, tj = torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()
    for layout in LAYOUTS:
        print(f"  {layout} ...", flush=True)
        x = a_d.t().contiguous() if layout == "TN" else a_d
        y = b_d.t().contiguous() if layout == "NT" else b_d
        assert "edge" not in B.plan_name(n, n, n, layout, now=True) and B.plan_name(n, n, n, layout, now=True) != "naive"
        c.view(torch.int16).fill_(0x7FC0)
        B.axonn_linear_fwd(n, n, n, layout, x, y, c)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(c.view(-1)[:: 4099].float()).all()), "unwritten or non-finite output"
        got = U.to_host_bits(c[ti, tj])
        U.assert_close(got, ref, f"square {n} {layout}")
        del x, y


# ------------------------------------------------------------------ shard shapes of the paper's model table
def _zoo_cases():
    """A seeded subset of the shard shapes of the paper's GPT models (Sec. V-A, model table: hidden 5120,
    7168, 9216, 12288 are the ones that are not powers of two; QKV 3h, FFN 4h) with both weight
    dimensions split by 1, 2, 4 or 8 (Sec. IV-A): per hidden size three (layer, split) choices whose
    weight shard stays below 2^25 elements, 2048 tokens."""
    rng = np.random.default_rng(2502)
    cases = []
    for h in (5120, 7168, 9216, 12288):
        layers = [("qkv", h, 3 * h), ("attn_out", h, h), ("fc1", h, 4 * h), ("fc2", 4 * h, h)]
        pool = [(nm, di // ga, do // gb) for nm, di, do in layers for ga in (1, 2, 4, 8) for gb in (1, 2, 4, 8)
                if (di // ga) * (do // gb) <= (1 << 25)]
        for k in rng.choice(len(pool), size=3, replace=False):
            cases.append((h,) + pool[int(k)])
    return cases


@pytest.mark.parametrize("h,layer,d_in,d_out", _zoo_cases())
def test_model_zoo_shard_shapes_sampled(oracle_mod, h, layer, d_in, d_out):
    """Forward, backward-data and backward-weight of a shard in their natural modes, automatic plan
    (what the model-zoo sweep times), on sampled rows, columns and one element per 128 x 128 block."""
    tokens = 2048
    t = synth.fc_layer_tensors(tokens, d_in, d_out, synth.BASE_SEED + 600 + h)
    for g in synth.fc_layer_gemms(tokens, d_in, d_out, f"h{h}.{layer}"):
        M, N, K = g["M"], g["N"], g["K"]
        ii, jj = _sample_positions(M, N, seed=M + N + K)
        A, Bm = synth.operands_for(g["op"], g["layout"], t)
        ref = oracle_mod.gemm_at(M, N, K, g["layout"], A, Bm, ii, jj)
        got = run_gpu(g["op"], M, N, K, g["layout"], A, Bm)
        assert np.isfinite(U.bits_to_f64(got)).all(), f"{g['name']}: unwritten or non-finite output"
        U.assert_close(got[ii, jj], ref, f"{g['name']} {g['layout']} {B.plan_name(M, N, K, g['layout'])}")


def _random_shapes():
    """Seeded shapes off the beaten track: tile counts that are odd, not multiples of 8, or one and a
    fraction rounds; outputs narrow in one direction over a long K; M and N multiples of 128, K of 64."""
    rng = np.random.default_rng(81450)
    cases = []
    for layout in LAYOUTS:
        for _ in range(7):
            narrow = rng.random() < 0.4
            M = int(rng.integers(1, 40)) * 128
            N = int(rng.integers(1, 12 if narrow else 40)) * 128
            if rng.random() < 0.5:
                M, N = N, M
            K = int(rng.integers(2, 300 if narrow else 96)) * 64
            cases.append((layout, M, N, K))
    return cases


@pytest.mark.parametrize("layout,M,N,K", _random_shapes())
def test_random_shapes_integer_data_sampled_bit_for_bit(oracle_mod, layout, M, N, K):
    """Automatic plan on seeded random shapes, small-integer data (every partial sum exact in fp32, so the
    result does not depend on how K is cut up or in which order partial tiles are added): sampled rows,
    columns and one element per 128 x 128 block must equal the oracle's bf16 rounding bit for bit."""
    a = synth.integer_bf16(7000 + M + K, (M, K), -3, 3)
    b = synth.integer_bf16(7001 + N + K, (K, N), -3, 3)
    A, Bm = store(a, b, layout)
    ii, jj = _sample_positions(M, N, seed=M * 7 + N * 3 + K)
    want = U.f64_to_bf16_bits_rne(oracle_mod.gemm_at(M, N, K, layout, A, Bm, ii, jj))
    got = run_gpu("fwd", M, N, K, layout, A, Bm)
    bad = np.flatnonzero(got[ii, jj] != want)
    assert bad.size == 0, (f"{layout} {M}x{N}x{K} plan {B.plan_name(M, N, K, layout)}: {bad.size} sampled outputs differ, "
                           f"first at ({ii[bad[0]]}, {jj[bad[0]]})")
    assert B.axonn_linear_split_k_timeouts() == 0


def test_model_zoo_plans_with_odd_split_counts_and_two_launches(oracle_mod):
    """Among the model-zoo shard shapes the planner picks split-K with 3, 5 and 6 K ranges (7 is never
    chosen there; test_every_tile_variant_against_oracle covers it) and plans of two launches: one
    product of each kind is found by scanning the plans (host logic) and checked on sampled outputs,
    N(0,1) data and integer data."""
    tokens = 2048
    wanted = {"_sk3": None, "_sk5": None, "_sk6": None, "+": None}
    for h in (5120, 7168, 9216, 12288, 4096, 16384):
        for nm, di, do in (("qkv", h, 3 * h), ("attn_out", h, h), ("fc1", h, 4 * h), ("fc2", 4 * h, h)):
            for ga in (1, 2, 4, 8):
                for gb in (1, 2, 4, 8):
                    d_in, d_out = di // ga, do // gb
                    if d_in * d_out > (5 << 23):
                        continue
                    for g in synth.fc_layer_gemms(tokens, d_in, d_out, f"h{h}.{nm}/{ga}x{gb}"):
                        name = B.plan_name(g["M"], g["N"], g["K"], g["layout"])
                        for key in wanted:
                            hit = key in name if key == "+" else name.endswith(key) and "+" not in name
                            if wanted[key] is None and hit:
                                wanted[key] = (g, d_in, d_out, name)
    assert all(v is not None for v in wanted.values()), {k: v for k, v in wanted.items() if v is None}
    for key, (g, d_in, d_out, name) in wanted.items():
        M, N, K = g["M"], g["N"], g["K"]
        print(f"  {key}: {g['name']} {g['layout']} {M}x{N}x{K} {name}", flush=True)
        ii, jj = _sample_positions(M, N, seed=M + K)
        for kind in ("normal", "integer"):
            if kind == "normal":
                t = synth.fc_layer_tensors(tokens, d_in, d_out, synth.BASE_SEED + 650)
            else:
                t = dict(X=synth.integer_bf16(synth.BASE_SEED + 660, (tokens, d_in), -4, 4),
                         W=synth.integer_bf16(synth.BASE_SEED + 661, (d_in, d_out), -4, 4),
                         dY=synth.integer_bf16(synth.BASE_SEED + 662, (tokens, d_out), -4, 4))
            A, Bm = synth.operands_for(g["op"], g["layout"], t)
            ref = oracle_mod.gemm_at(M, N, K, g["layout"], A, Bm, ii, jj)
            got = run_gpu(g["op"], M, N, K, g["layout"], A, Bm)
            assert np.isfinite(U.bits_to_f64(got)).all(), f"{name}: unwritten or non-finite output"
            if kind == "normal":
                U.assert_close(got[ii, jj], ref, f"{g['name']} {name}")
            else:
                assert np.array_equal(got[ii, jj], U.f64_to_bf16_bits_rne(ref)), f"{g['name']} {name}: integer data"
    assert B.axonn_linear_split_k_timeouts() == 0


# ------------------------------------------------------------------ products cut into two launches
@pytest.mark.parametrize("shape", [(2048, 10240, 1024), (2560, 8192, 1024)])
@pytest.mark.parametrize("layout", LAYOUTS)
def test_two_launch_plans_every_element(oracle_mod, layout, shape):
    """Outputs of one and a quarter rounds of large tiles: the library cuts off the last columns
    (first shape) or the last rows (second shape) into a launch of their own; every element checked."""
    M, N, K = shape
    parts = B.plan(M, N, K, layout)
    assert len(parts) == 2, parts
    assert (parts[1]["col0"] > 0) == (shape[1] == 10240) and (parts[1]["row0"] > 0) == (shape[0] == 2560)
    a = synth.normal_bf16(synth.BASE_SEED + 700, (M, K))
    b = synth.normal_bf16(synth.BASE_SEED + 701, (K, N))
    A, Bm = store(a, b, layout)
    ref = oracle_mod.gemm(M, N, K, layout, A, Bm)
    got = run_gpu("fwd", M, N, K, layout, A, Bm)
    U.assert_close(got, ref, f"two launches {shape} {layout}")
    # integer-valued operands: bit for bit, whichever launch wrote the element
    ai = synth.integer_bf16(synth.BASE_SEED + 702, (M, K), -4, 4)
    bi = synth.integer_bf16(synth.BASE_SEED + 703, (K, N), -4, 4)
    A, Bm = store(ai, bi, layout)
    got = run_gpu("fwd", M, N, K, layout, A, Bm)
    assert np.array_equal(got, U.f64_to_bf16_bits_rne(oracle_mod.gemm(M, N, K, layout, A, Bm)))


@pytest.mark.parametrize("shape", [(2048, 12288, 8192), (12288, 2048, 8192), (2048, 4608, 18432)])
def test_two_launch_plan_with_split_k_block_sampled(oracle_mod, shape):
    """One round and a half of large tiles at a long K: the second block runs as split-K (NT),
    reading its operands and writing its output through the whole matrices' leading dimensions.
    Third shape: 144 large tiles, less than a round; both blocks run as split-K, one after the
    other through the same scratch area."""
    M, N, K = shape
    parts = B.plan(M, N, K, "NT")
    assert len(parts) == 2 and splits_of(parts[1]["variant"]) > 1, parts
    a = synth.normal_bf16(synth.BASE_SEED + 710, (M, K))
    b = synth.normal_bf16(synth.BASE_SEED + 711, (K, N))
    ii, jj = _sample_positions(M, N, seed=M + 7)
    ref = oracle_mod.gemm_at(M, N, K, "NN", a, b, ii, jj)
    for layout in LAYOUTS:
        A, Bm = store(a, b, layout)
        got = run_gpu("fwd", M, N, K, layout, A, Bm)
        assert np.isfinite(U.bits_to_f64(got)).all(), f"{shape} {layout}: unwritten or non-finite output"
        U.assert_close(got[ii, jj], ref, f"two launches, split-K block {shape} {layout}")


def test_long_k_four_ranges_full_chip_sampled(oracle_mod):
    """64 large tiles at K = 32768: four K ranges per tile on all 256 compute units, one range per
    pair of XCDs (the configuration the shard shapes of the widest models run in)."""
    M, N, K = 2048, 2048, 32768
    assert all(B.plan_name(M, N, K, lay).endswith("_sk4") for lay in LAYOUTS)
    a = synth.normal_bf16(synth.BASE_SEED + 720, (M, K))
    b = synth.normal_bf16(synth.BASE_SEED + 721, (K, N))
    ii, jj = _sample_positions(M, N, seed=K)
    ref = oracle_mod.gemm_at(M, N, K, "NN", a, b, ii, jj)
    for layout in LAYOUTS:
        A, Bm = store(a, b, layout)
        got = run_gpu("bwd_data", M, N, K, layout, A, Bm)
        assert np.isfinite(U.bits_to_f64(got)).all()
        U.assert_close(got[ii, jj], ref, f"long K, four ranges {layout}")
    assert B.axonn_linear_split_k_timeouts() == 0


def test_panel_larger_than_4_gib(oracle_mod):
    """An MN-contiguous operand of 6 GiB (TN: A stored [K, M] with M = 98304, K = 32768): the K window
    of its direct loads must move in 64-bit pointers (32-bit per-lane offsets would wrap after 21845
    k-rows and every output element would be wrong).  A is a seeded 1024-row block repeated along
    k (the wrap lands a third of a row off, so periodic data still shows it); integer data, sampled
    outputs compared bit for bit."""
    M, N, K = 98304, 256, 32768
    block = synth.integer_bf16(synth.BASE_SEED + 730, (1024, M), -4, 4)
    A = np.tile(block, (K // 1024, 1))                       # [K, M]
    Bm = synth.integer_bf16(synth.BASE_SEED + 731, (K, N), -4, 4)
    assert A.shape == (K, M) and A.nbytes > (1 << 32)
    rng = np.random.default_rng(730)
    ii = rng.integers(0, M, 96).astype(np.int64)
    jj = rng.integers(0, N, 96).astype(np.int64)
    want = U.f64_to_bf16_bits_rne(oracle_mod.gemm_at(M, N, K, "TN", A, Bm, ii, jj))
    for v in (-1, [B.variant_name(x) for x in range(B.num_variants())].index("mfma16k64_256x256_w8"),
              [B.variant_name(x) for x in range(B.num_variants())].index("mfma16_256x256_w8")):
        got = run_gpu("bwd_weight", M, N, K, "TN", A, Bm, variant=v)
        assert np.array_equal(got[ii, jj], want), f"variant {v}"


# ------------------------------------------------------------------ operand re-storage (transpose)
@pytest.mark.parametrize("shape", [(64, 64), (128, 192), (4096, 1024), (2048, 12288), (1, 7), (65, 130),
                                   (257, 31), (64, 72), (1000, 8)])
def test_transpose_matches_oracle_bit_for_bit(oracle_mod, shape):
    rows, cols = shape
    # position-coded values (every element differs from its neighbours) XOR seeded noise
    src = ((np.arange(rows, dtype=np.int64)[:, None] * 251 + np.arange(cols, dtype=np.int64)[None, :] * 7) % 65521)
    src = (src.astype(np.uint16)) ^ synth.normal_bf16(77, (rows, cols))
    want = oracle_mod.transpose(src)
    s = U.to_device(src)
    d = torch.empty((cols, rows), dtype=torch.bfloat16, device="cuda")
    d.view(torch.int16).fill_(0x7FC0)
    B.axonn_transpose_bf16(rows, cols, s, d)
    torch.cuda.synchronize()
    got = U.to_host_bits(d)
    assert np.array_equal(got, want), f"first mismatch at {np.argwhere(got != want)[:1]}"
    assert np.array_equal(U.to_host_bits(s), src)   # the source is untouched


def test_transposed_weight_runs_the_forward_product_in_another_mode(oracle_mod):
    # Sec. IV-C in one piece: Y = X W computed as NN on (X, W) and as NT on (X, transpose(W))
    T, d_in, d_out = 512, 768, 1024
    t = synth.fc_layer_tensors(T, d_in, d_out, synth.BASE_SEED + 700)
    ref = oracle_mod.gemm(T, d_out, d_in, "NN", t["X"], t["W"])
    X, W = U.to_device(t["X"]), U.to_device(t["W"])
    Wt = torch.empty((d_out, d_in), dtype=torch.bfloat16, device="cuda")
    B.axonn_transpose_bf16(d_in, d_out, W, Wt)
    y_nn = torch.empty((T, d_out), dtype=torch.bfloat16, device="cuda")
    y_nt = torch.empty_like(y_nn)
    B.axonn_linear_fwd(T, d_out, d_in, "NN", X, W, y_nn)
    B.axonn_linear_fwd(T, d_out, d_in, "NT", X, Wt, y_nt)
    torch.cuda.synchronize()
    U.assert_close(U.to_host_bits(y_nn), ref, "fwd NN")
    U.assert_close(U.to_host_bits(y_nt), ref, "fwd NT on the transposed weight")


# ------------------------------------------------------------------ mode tuner (Sec. IV-C)
@pytest.mark.parametrize("op", ["fwd", "bwd_data", "bwd_weight"])
def test_tuner_times_all_modes_and_leaves_the_right_product(oracle_mod, op):
    T, d_in, d_out = 512, 768, 1024
    t = synth.fc_layer_tensors(T, d_in, d_out, synth.BASE_SEED + 800)
    g = next(x for x in synth.fc_layer_gemms(T, d_in, d_out, "fc") if x["op"] == op)
    M, N, K, nat = g["M"], g["N"], g["K"], g["layout"]
    A, Bm = synth.operands_for(op, nat, t)
    ref = oracle_mod.gemm(M, N, K, nat, A, Bm)
    a, b = U.to_device(A), U.to_device(Bm)
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    c.view(torch.int16).fill_(0x7FC0)
    scratch = torch.empty(((M * K * 2 + 255) // 256 * 256 + K * N * 2,), dtype=torch.uint8, device="cuda")
    B.axonn_linear_tune_reset()
    res = B.axonn_linear_tune(op, M, N, K, a, b, c, scratch)
    torch.cuda.synchronize()
    assert all(us > 0 for us in res["gemm_us"]), res
    assert res["best_layout"] == int(np.argmin(res["gemm_us"]))
    nat_i = B.LAYOUTS[nat]
    assert res["restore_first_us"][nat_i] == 0 and res["restore_second_us"][nat_i] == 0
    for m in range(3):   # a mode pays for exactly the operands it wants stored the other way
        assert (res["restore_first_us"][m] > 0) == ((m != 2) != (nat_i != 2))
        assert (res["restore_second_us"][m] > 0) == ((m != 1) != (nat_i != 1))
    # the last mode timed (TN) ran on re-stored operands unless TN is the natural mode: its output
    # is the product all the same
    U.assert_close(U.to_host_bits(c), ref, f"tuner output {op}")
    assert B.axonn_linear_tuned(op, M, N, K) == res
    # without scratch only the natural mode can be tried, and it wins
    B.axonn_linear_tune_reset()
    res0 = B.axonn_linear_tune(op, M, N, K, a, b, c, None)
    assert res0["best_layout"] == nat_i and sorted(us > 0 for us in res0["gemm_us"]) == [False, False, True]


@pytest.mark.parametrize("op", ["fwd", "bwd_data", "bwd_weight"])
def test_tuned_call_runs_the_product_in_the_remembered_mode(oracle_mod, op):
    """Sec. IV-C, second half: once a mode has been chosen for a product it is the mode that runs.  Every
    mode is set as the remembered winner in turn; the call re-stores what that mode wants transposed (the
    first operand per call, the second from a copy the caller holds, or per call when it holds none) and
    the output is the product all the same."""
    T, d_in, d_out = 512, 768, 1024
    t = synth.fc_layer_tensors(T, d_in, d_out, synth.BASE_SEED + 810)
    g = next(x for x in synth.fc_layer_gemms(T, d_in, d_out, "fc") if x["op"] == op)
    M, N, K, nat = g["M"], g["N"], g["K"], g["layout"]
    A, Bm = synth.operands_for(op, nat, t)
    ref = oracle_mod.gemm(M, N, K, nat, A, Bm)
    a, b = U.to_device(A), U.to_device(Bm)
    b_t = torch.empty((Bm.shape[1], Bm.shape[0]), dtype=torch.bfloat16, device="cuda")
    B.axonn_transpose_bf16(Bm.shape[0], Bm.shape[1], b, b_t)       # the copy a caller would hold of a weight
    scratch = torch.empty(((M * K * 2 + 255) // 256 * 256 + K * N * 2,), dtype=torch.uint8, device="cuda")
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    B.axonn_linear_tune_reset()
    try:
        c.view(torch.int16).fill_(0x7FC0)
        assert B.axonn_linear_tuned_call(op, M, N, K, a, b, c, None, scratch) == B.LAYOUTS[nat]   # not tuned: natural mode
        torch.cuda.synchronize()
        U.assert_close(U.to_host_bits(c), ref, f"untuned {op}")
        for mode in LAYOUTS:
            B.axonn_linear_tuned_set(op, M, N, K, mode)
            assert B.axonn_linear_tuned(op, M, N, K)["best_layout_all_in"] == B.LAYOUTS[mode]
            for held in (b_t, None):
                c.view(torch.int16).fill_(0x7FC0)
                used = B.axonn_linear_tuned_call(op, M, N, K, a, b, c, held, scratch)
                torch.cuda.synchronize()
                assert used == B.LAYOUTS[mode], (op, mode, used)
                U.assert_close(U.to_host_bits(c), ref, f"tuned {op} in {mode}, held copy {held is not None}")
            # no room to re-store: the natural mode runs, unless the held copy is all that mode needs
            c.view(torch.int16).fill_(0x7FC0)
            used = B.axonn_linear_tuned_call(op, M, N, K, a, b, c, b_t, None)
            torch.cuda.synchronize()
            needs_first = (mode == "TN") != (nat == "TN")
            assert used == (B.LAYOUTS[nat] if needs_first else B.LAYOUTS[mode])
            U.assert_close(U.to_host_bits(c), ref, f"tuned {op} in {mode}, no scratch")
        assert np.array_equal(U.to_host_bits(a), A) and np.array_equal(U.to_host_bits(b), Bm)   # operands untouched
    finally:
        B.axonn_linear_tune_reset()
