"""Shape sweeps of the FC-layer GEMMs on one MI355X (timing only; parity is the tests' job).

    python -m paper_2502_08145_amd.sweeps peak_curve [--max 65536]
    python -m paper_2502_08145_amd.sweeps model_zoo [--tokens 2048]
    python -m paper_2502_08145_amd.sweeps variant_eff [--hot]

peak_curve   square bf16 GEMMs 1024 ... 65536 in the three modes, the protocol of the paper's
             single-GPU GEMM benchmark (Sec. V-C: repeated runs, mean of the last three quarters),
             with the repetition count scaled down so that one size takes a few seconds.
model_zoo    the shard shapes of the paper's model table (Sec. V-A, the table of GPT models: hidden 4096 ... 16384,
             FFN 4h, fused QKV 3h) under every split of a weight's two dimensions by 1, 2, 4 or 8
             (Sec. IV-A: a weight is sharded over two of the grid's dimensions), forward,
             backward-data and backward-weight in their natural modes.

variant_eff  every kernel variant without split-K, forced, on benchmark-like shapes in all three modes,
             operands cycling through sets larger than the Infinity Cache; prints the throughputs in
             units of 1200 TFLOP/s, which is what the library's selection model keeps per variant
             (Variant::eff in csrc/axonn_linear.hip).

Operands are N(0,1) (activations, gradients) and N(0, 0.02^2) (weights) drawn on the device with a
fixed seed: host generation of 65536^2 matrices would take minutes.  Output: one text line per
GEMM / per hidden size on stdout.
"""
from __future__ import annotations

import argparse
import re
import subprocess
import sys

import torch

from . import binding as B

PEAK = 2516.6


def time_gemm(op, M, N, K, layout, a, b, c, reps, warm=3):
    stream = torch.cuda.current_stream()
    for _ in range(warm):
        B.OPS[op](M, N, K, layout, a, b, c, 1, stream)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    ev[0].record(stream)
    for i in range(reps):
        B.OPS[op](M, N, K, layout, a, b, c, 1, stream)
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    t = [ev[i].elapsed_time(ev[i + 1]) for i in range(reps)]
    tail = t[len(t) // 4:]            # mean of the last three quarters
    return sum(tail) / len(tail)      # ms


def randn_bf16(shape, sigma, gen):
    return (torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * sigma).to(torch.bfloat16)


def peak_curve(args):
    gen = torch.Generator(device="cuda").manual_seed(250208145)
    n = 1024
    print(f"{'n':>6s} {'mode':>4s} {'variant':<22s} {'reps':>4s} {'ms':>10s} {'TFLOP/s':>9s} {'% peak':>7s}")
    while n <= args.max:
        a = randn_bf16((n, n), 1.0, gen)
        b = randn_bf16((n, n), 1.0, gen)
        c = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
        for layout in ("NN", "NT", "TN"):
            est = 2.0 * n ** 3 / 1.0e15 * 1e3            # ms at 1 PFLOP/s
            reps = int(max(4, min(100, 2000.0 / max(est, 1e-3))))
            ms = time_gemm("fwd", n, n, n, layout, a, b, c, reps)
            tf = 2.0 * n ** 3 / ms / 1e9
            v = B.plan_name(n, n, n, layout)
            print(f"{n:6d} {layout:>4s} {v:<22s} {reps:4d} {ms:10.4f} {tf:9.1f} {tf / PEAK * 100:6.1f}%", flush=True)
        del a, b, c
        n *= 2


def model_zoo(args):
    gen = torch.Generator(device="cuda").manual_seed(250208146)
    T = args.tokens
    splits = (1, 2, 4, 8)
    print(f"tokens per GPU {T}; per hidden size: all 16 splits x 4 layers x 3 products")
    print(f"{'hidden':>6s} {'GEMMs':>5s} {'guarded':>7s} {'min':>8s} {'median':>8s} {'max':>8s} {'aggregate':>9s}  slowest shape")
    for h in (4096, 5120, 7168, 9216, 12288, 16384):
        layers = [("qkv", h, 3 * h), ("attn_out", h, h), ("fc1", h, 4 * h), ("fc2", 4 * h, h)]
        rates, flops_sum, ms_sum, guarded, worst = [], 0.0, 0.0, 0, None
        for name, d_in, d_out in layers:
            for ga in splits:
                for gb in splits:
                    di, do = d_in // ga, d_out // gb
                    X = randn_bf16((T, di), 1.0, gen)
                    W = randn_bf16((di, do), 0.02, gen)
                    dY = randn_bf16((T, do), 1.0, gen)
                    for op, lay, M, N, K, p, q in (("fwd", "NN", T, do, di, X, W), ("bwd_data", "NT", T, di, do, dY, W),
                                                   ("bwd_weight", "TN", di, do, T, X, dY)):
                        c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
                        v = B.select_variant(M, N, K, lay)
                        guarded += v == 0 or v == B.num_variants() - 1     # naive or guarded MFMA kernel
                        ms = time_gemm(op, M, N, K, lay, p, q, c, 12 if v else 3, warm=2)
                        fl = 2.0 * M * N * K
                        tf = fl / ms / 1e9
                        rates.append(tf)
                        flops_sum += fl
                        ms_sum += ms
                        if worst is None or tf < worst[0]:
                            worst = (tf, f"{name}.{op} {lay} M={M} N={N} K={K} {B.plan_name(M, N, K, lay)}")
                        if args.verbose:
                            print(f"   {h} {name}.{op} {lay} M={M} N={N} K={K} {B.plan_name(M, N, K, lay)} {ms * 1e3:.1f} us {tf:.0f}", flush=True)
                    del X, W, dY
        rates.sort()
        print(f"{h:6d} {len(rates):5d} {guarded:7d} {rates[0]:8.1f} {rates[len(rates) // 2]:8.1f} {rates[-1]:8.1f} "
              f"{flops_sum / ms_sum / 1e9:9.1f}  {worst[1]} ({worst[0]:.0f} TFLOP/s)", flush=True)


def variant_eff(args):
    """Efficiencies of the selection model: mean over the shapes of TFLOP/s / 1200, per variant and mode.
    Every launch takes the next of several operand sets that together exceed the 256 MB Infinity Cache
    three times, so the rates are those of operands coming from HBM, as in a training step."""
    gen = torch.Generator(device="cuda").manual_seed(250208148)
    # outputs that fill the 256 compute units a whole number of times with every tile shape (a partly
    # filled round is the selection model's own term)
    shapes = [(4096, 4096, 4096), (4096, 16384, 2048), (2048, 16384, 4096), (4096, 8192, 8192)]
    names = [B.variant_name(v) for v in range(B.num_variants())]
    stream = torch.cuda.current_stream()
    rows = {}
    for M, N, K in shapes:
        sets = 1 if args.hot else max(2, -(-(768 << 20) // (2 * (M * K + K * N + M * N))))
        a = [randn_bf16((M, K), 1.0, gen) for _ in range(sets)]
        b = [randn_bf16((K, N), 1.0, gen) for _ in range(sets)]
        c = [torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for _ in range(sets)]
        for layout in ("NN", "NT", "TN"):
            x = [t.t().contiguous() for t in a] if layout == "TN" else a
            y = [t.t().contiguous() for t in b] if layout == "NT" else b
            for v, name in enumerate(names):
                if v == 0 or "_sk" in name or "edge" in name or not B.variant_supports(v, M, N, K, layout):
                    continue
                B.force_variant(v)
                try:
                    reps = max(12, 4 * sets)
                    for i in range(sets):
                        B.axonn_linear_fwd(M, N, K, layout, x[i], y[i], c[i], 1, stream)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for i in range(reps):
                        B.axonn_linear_fwd(M, N, K, layout, x[i % sets], y[i % sets], c[i % sets], 1, stream)
                    e1.record(stream)
                    torch.cuda.synchronize()
                    ms = e0.elapsed_time(e1) / reps
                finally:
                    B.force_variant(-1)
                tf = 2.0 * M * N * K / ms / 1e9
                rows.setdefault(name, {}).setdefault(layout, []).append(tf)
                print(f"{M:6d} {N:6d} {K:6d} {layout} {name:<24s} {sets:3d} sets {ms * 1e3:9.1f} us {tf:8.1f} TFLOP/s", flush=True)
            del x, y
        del a, b, c
    print("variant                    eff NN   NT   TN   (TFLOP/s / 1200, mean over the shapes)")
    for name, d in rows.items():
        # a variant may exist for one mode only
        e = [f"{sum(d[l]) / len(d[l]) / 1200.0:4.2f}" if l in d else "   -" for l in ("NN", "NT", "TN")]
        print(f"{name:<26s}   {e[0]} {e[1]} {e[2]}")


def parse_smi(text):
    """(socket power in W or None, [shader clock of each XCD in MHz]) from the text of `amd-smi metric -c -p`."""
    power = re.search(r"SOCKET_POWER:\s*(\d+)\s*W", text)
    clocks = [int(m) for m in re.findall(r"GFX_\d+:\s*\n\s*CLK:\s*(\d+)\s*MHz", text)]
    return (int(power.group(1)) if power else None), clocks


def smi_sample():
    """Power and shader clocks as amd-smi prints them right now."""
    return parse_smi(subprocess.run(["amd-smi", "metric", "-c", "-p"], capture_output=True, text=True, timeout=30).stdout)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    p = sub.add_parser("peak_curve")
    p.add_argument("--max", type=int, default=65536)
    z = sub.add_parser("model_zoo")
    z.add_argument("--tokens", type=int, default=2048)
    z.add_argument("--verbose", action="store_true")
    e = sub.add_parser("variant_eff")
    e.add_argument("--hot", action="store_true", help="one operand set, re-used by every launch (operands stay in cache)")
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("sweeps: no GPU visible")
    B.lib()
    torch.cuda.set_device(0)
    B.register_workspace()          # the library allocates nothing: split-K scratch is ours to provide
    {"peak_curve": peak_curve, "model_zoo": model_zoo, "variant_eff": variant_eff}[args.cmd](args)


if __name__ == "__main__":
    main()
