#!/usr/bin/env python3
"""What the matrix pipe alone sustains, as a function of the operand values (pd_mfma_probe).

    python3 -m paper_2603_04716_amd.mfma_ceiling_probe

256 workgroups of 8 waves issue nothing but v_mfma_f32_32x32x16_bf16 on register operands.  The
operand patterns go from the cheapest for the hardware (all ones) to the benchmark's own values:
A fragments drawn like the layer's weights (N(0, 0.02^2), bf16) and B fragments like its hidden
states (N(0, 1), bf16).  Prints a markdown table: pattern, milliseconds, PFLOP/s, fraction of the
published 2.5 PFLOP/s bf16 peak.  The last row is the ceiling the prefill GEMMs are measured against
beside the published peak.
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

N_WG, ITERS, PEAK = 256, 200000, 2.5e15


NA, NB = 16384, 8192                # bf16 elements of the A and B fragments of one workgroup


def _dev(a):
    import numpy as np
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda().to(torch.bfloat16).contiguous()


def sustained_tflops(a_vals, b_vals, iters=ITERS, reps=7, warmup=2):
    """TFLOP/s of the register-only loop on the given operand values (median of `reps` launches)."""
    import numpy as np
    import torch
    import paper_2603_04716_amd as pd
    ad, bd = _dev(a_vals), _dev(b_vals)
    sink = torch.empty(N_WG * 512, dtype=torch.float32, device="cuda")
    flops = 2.0 * 32 * 32 * 16 * 8 * iters * 8 * N_WG
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ts = []
    for rep in range(warmup + reps):
        e0.record()
        pd.pd_mfma_probe(ad, bd, N_WG, iters, sink)
        e1.record()
        e1.synchronize()
        if rep >= warmup:
            ts.append(e0.elapsed_time(e1))
    return flops / (float(np.median(ts)) * 1e-3) / 1e12


def benchmark_operands(seed=0):
    """A fragments drawn like the layer's weights, B fragments like its hidden states."""
    import numpy as np
    rng = np.random.default_rng(seed)
    return 0.02 * rng.standard_normal(NA), rng.standard_normal(NB)


def main():
    import numpy as np
    import torch
    import paper_2603_04716_amd as pd

    rng = np.random.default_rng(0)
    dev = _dev
    na, nb = NA, NB
    patterns = [
        ("all ones", np.ones(na), np.ones(nb)),
        ("zeros", np.zeros(na), np.zeros(nb)),
        ("positive, random mantissa in [1, 2)", 1 + rng.random(na), 1 + rng.random(nb)),
        ("random sign, random mantissa in [1, 2)", (1 + rng.random(na)) * rng.choice([-1, 1], na),
         (1 + rng.random(nb)) * rng.choice([-1, 1], nb)),
        ("N(0, 1) x N(0, 1)", rng.standard_normal(na), rng.standard_normal(nb)),
        ("weights N(0, 0.02^2) x hidden states N(0, 1)  (the benchmark's operands)",
         0.02 * rng.standard_normal(na), rng.standard_normal(nb)),
    ]
    sink = torch.empty(N_WG * 512, dtype=torch.float32, device="cuda")
    flops = 2.0 * 32 * 32 * 16 * 8 * ITERS * 8 * N_WG
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    print(f"{N_WG} workgroups x 8 waves x {ITERS} x 8 v_mfma_f32_32x32x16_bf16 = {flops / 1e12:.1f} TFLOP per launch")
    print()
    print("| operand values | ms (median of 7) | PFLOP/s | of 2.5 PFLOP/s |")
    print("|---|---|---|---|")
    for name, a, b in patterns:
        ad, bd = dev(a), dev(b)
        ts = []
        for rep in range(9):
            e0.record()
            pd.pd_mfma_probe(ad, bd, N_WG, ITERS, sink)
            e1.record()
            e1.synchronize()
            if rep >= 2:
                ts.append(e0.elapsed_time(e1))
        ms = float(np.median(ts))
        print(f"| {name} | {ms:.2f} | {flops / (ms * 1e-3) / 1e15:.3f} | {flops / (ms * 1e-3) / PEAK:.3f} |", flush=True)


if __name__ == "__main__":
    main()
