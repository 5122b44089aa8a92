"""The entry point for callers that cannot allocate: axonn_linear_gemm_static runs the split-K kernels
through the library's static device array.  Its output must equal, bit for bit, what the ordinary entry
point gives with a registered workspace (same kernels, same fixed summation order), on two calls in a
row, the second on a smaller input; and both must match the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2502_08145_amd import binding as B
from paper_2502_08145_amd import synth
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _product(op, M, N, K, layout, seed, integer):
    if integer:
        a = synth.integer_bf16(seed, (M, K), -4, 4)
        b = synth.integer_bf16(seed + 1, (K, N), -4, 4)
    else:
        a = synth.normal_bf16(seed, (M, K))
        b = synth.normal_bf16(seed + 1, (K, N), 0.02)
    A = a if layout != "TN" else synth.transpose_bits(a)
    Bm = b if layout != "NT" else synth.transpose_bits(b)
    return a, b, A, Bm


def test_static_scratch_entry_point_matches_the_registered_workspace_path(oracle_mod):
    print("\n[gpu-test] static scratch entry point", flush=True)
    assert B.axonn_linear_static_scratch_bytes() == 4096 + 128 * 256 * 256 * 4
    U.shared_workspace()
    # first call: 128 large tiles, two K ranges (the whole static area); second, right behind it on the
    # same stream and smaller: 64 small tiles, two K ranges; a third that needs no scratch at all
    cases = [("bwd_data", 2048, 4096, 8192, "NT", False), ("fwd", 1024, 1024, 8192, "NN", True),
             ("bwd_weight", 512, 768, 448, "TN", False)]
    names = [B.plan_name(M, N, K, lay, now=True) for _, M, N, K, lay, _ in cases]
    assert names[0].endswith("_sk2") and "_sk" in names[1] and "_sk" not in names[2], names
    dev_in, outs_static, outs_ws, hosts = [], [], [], []
    for i, (op, M, N, K, lay, integer) in enumerate(cases):
        a, b, A, Bm = _product(op, M, N, K, lay, 4100 + 10 * i, integer)
        hosts.append((a, b))
        dev_in.append((U.to_device(A), U.to_device(Bm)))
        outs_static.append(torch.empty((M, N), dtype=torch.bfloat16, device="cuda"))
        outs_ws.append(torch.empty((M, N), dtype=torch.bfloat16, device="cuda"))
    for c in outs_static + outs_ws:
        c.view(torch.int16).fill_(0x7FC0)
    B.axonn_linear_init()      # code object loaded (the static array comes with it), its address looked up
    for rnd in range(2):       # the calls back to back, no synchronisation in between; then once more
        if rnd == 1:
            # steady state (the HIP runtime sets up its own launch resources during the first launches
            # of a process): from here on the free device memory must not move
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info()[0]
        for (op, M, N, K, lay, _), (x, y), c in zip(cases, dev_in, outs_static):
            B.axonn_linear_gemm_static(M, N, K, lay, x, y, c)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated"
    for (op, M, N, K, lay, _), (x, y), c in zip(cases, dev_in, outs_ws):
        B.OPS[op](M, N, K, lay, x, y, c)
    torch.cuda.synchronize()
    for (op, M, N, K, lay, integer), (a, b), cs, cw in zip(cases, hosts, outs_static, outs_ws):
        got, base = U.to_host_bits(cs), U.to_host_bits(cw)
        assert np.array_equal(got, base), f"{op} {M}x{N}x{K} {lay}: static-scratch result differs from the workspace path"
        ref = oracle_mod.gemm(M, N, K, "NN", a, b)
        if integer:
            assert np.array_equal(got, U.f64_to_bf16_bits_rne(ref))
        else:
            U.assert_close(got, ref, f"static {op} {lay}")
    # with no workspace registered the static entry point still splits; the ordinary one does not
    B.axonn_linear_set_workspace(None)
    try:
        op, M, N, K, lay, _ = cases[1]
        x, y = dev_in[1]
        c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        c.view(torch.int16).fill_(0x7FC0)
        B.axonn_linear_gemm_static(M, N, K, lay, x, y, c)
        torch.cuda.synchronize()
        assert np.array_equal(U.to_host_bits(c), U.to_host_bits(outs_ws[1]))
        # a plan beyond the static area is refused, and nothing is written
        M, N, K = 2048, 2048, 32768
        assert B.axonn_linear_workspace_bytes(M, N, K, "NT") > B.axonn_linear_static_scratch_bytes()
        xa = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
        xb = torch.zeros((N, K), dtype=torch.bfloat16, device="cuda")
        c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        c.view(torch.int16).fill_(0x7FC0)
        rc = B.axonn_linear_gemm_static(M, N, K, "NT", xa, xb, c, check=False)
        torch.cuda.synchronize()
        assert rc == B.AXONN_ERR_WORKSPACE and "static" in B.status_string(rc)
        assert bool((c.view(torch.int16) == 0x7FC0).all())
    finally:
        U.shared_workspace()
    assert B.axonn_linear_split_k_timeouts() == 0
