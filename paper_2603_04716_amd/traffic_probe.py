#!/usr/bin/env python3
"""HBM traffic of the layer's kernels from hardware counters, calibrated by a plain copy.

Run the workload under the profiler once per counter (from /tmp with TMPDIR=/tmp):

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d <dir>/fetch -o t -- \
        python3 -m paper_2603_04716_amd.traffic_probe
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d <dir>/write -o t -- \
        python3 -m paper_2603_04716_amd.traffic_probe

then summarise the two counter files:

    python3 -m paper_2603_04716_amd.traffic_probe --summarise <fetch csv> <write csv>

The workload is the 8B-shaped bf16 layer: a 1 GiB pd_stream_copy (known traffic: 1 GiB read and
1 GiB written), a prefill of 4 x 2048 tokens and a decode step of 256 sequences over 2048 cached
tokens, each three times.  A counter reads KiB per dispatch; the copy kernel's reading against its
known size gives the scale factor applied to every other kernel.

`--decode-batches 64,128,256` replaces the prefill / batch-256 pair by decode steps at the listed
batches (a kernel instance is told apart by its grid and workgroup size), and
`--durations <kernel trace csv>` prints the mean duration, workgroup count and workgroup size of
every (kernel, grid) of a `rocprofv3 --kernel-trace` run of the same workload, and
`--decode-steps <kernel trace csv> <fetch csv> <write csv>` lays the `--decode-batches` runs out step
by step: one row per launch of a decode step, with its workgroups, K splits, mean duration and
fetched / written bytes over the steps of that batch.
"""
import argparse
import collections
import csv
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

COPY_BYTES = 1 << 30
L_IN, N_SEQ, KV_LEN, BATCH = 2048, 4, 2048, 256


def workload(decode_batches=None):
    import torch
    import pd_inputs as I
    import paper_2603_04716_amd as pd
    from paper_2603_04716_amd import harness as H

    cfg = I.CONFIGS["llama8b"]
    layer = H.Layer(cfg, I.layer_weights(cfg))
    T = L_IN * N_SEQ
    x = H._dev(I.hidden(T, cfg["d_model"], seed=10, dtype="bf16"), "bf16")
    out = torch.empty_like(x)
    cu = [L_IN * i for i in range(N_SEQ + 1)]
    pd.pd_layer_reserve(layer.h, T)
    bmax = max(decode_batches) if decode_batches else BATCH
    cache = layer.new_cache(bmax, KV_LEN + 8)
    k, v = I.kv_fill(cfg["n_kv_heads"], KV_LEN, cfg["head_dim"], seed=11, dtype="bf16")
    layer.fill_cache(cache, [KV_LEN] * bmax, H._dev(k, "bf16"), H._dev(v, "bf16"))
    xdec = H._dev(I.hidden(bmax, cfg["d_model"], seed=12, dtype="bf16"), "bf16")
    odec = torch.empty_like(xdec)
    src = torch.ones(COPY_BYTES // 2, dtype=torch.bfloat16, device="cuda")
    dst = torch.empty_like(src)
    pd.pd_layer_reserve(layer.h, max(T, bmax))
    torch.cuda.synchronize()
    for _ in range(3):
        pd.pd_stream_copy(dst, src)
        if decode_batches:
            for B in decode_batches:
                for _rep in range(3):
                    pd.pd_kv_cache_set_lens(cache, list(range(B)), [KV_LEN] * B)
                    pd.pd_decode_step(layer.h, xdec[:B].contiguous(), list(range(B)), cache, odec[:B])
        else:
            pd.pd_prefill(layer.h, x, cu, out)
            pd.pd_kv_cache_set_lens(cache, list(range(BATCH)), [KV_LEN] * BATCH)
            pd.pd_decode_step(layer.h, xdec, list(range(BATCH)), cache, odec)
        torch.cuda.synchronize()
    layer.close()


def short(name):
    name = name.replace("void ", "").replace("pd::", "")
    cut = name.find("(")
    return name if cut < 0 else name[:cut]


def read_counter(path, counter):
    """{(kernel, grid): [KiB per dispatch]} for rows of `counter`."""
    agg = collections.defaultdict(list)
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            agg[(short(r["Kernel_Name"]), int(r["Grid_Size"]))].append(float(r["Counter_Value"]))
    return agg


def durations(trace_csv):
    """Mean duration per (kernel, grid) of a kernel-trace csv (columns of rocprofv3's kernel_trace)."""
    agg = collections.defaultdict(list)
    with open(trace_csv) as f:
        for r in csv.DictReader(f):
            wg = int(r["Workgroup_Size_X"]) * int(r.get("Workgroup_Size_Y", 1) or 1) * int(r.get("Workgroup_Size_Z", 1) or 1)
            grid = int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1) * int(r.get("Grid_Size_Z", 1) or 1)
            agg[(short(r["Kernel_Name"]), grid, wg)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    print("| kernel | workgroups | threads per workgroup | dispatches | mean us | min us |")
    print("|---|---|---|---|---|---|")
    for key in sorted(agg, key=lambda k: (k[0], k[1])):
        v = agg[key]
        print(f"| `{key[0]}` | {key[1] // key[2]} | {key[2]} | {len(v)} | {sum(v) / len(v):.1f} | {min(v):.1f} |")


def decode_steps(trace_csv, fetch_csv, write_csv):
    """The launches of one decode step, batch by batch.  A step starts at decode_meta_norm_kernel
    (its grid is batch + 1 workgroups) and ends at the last split-K sum or GEMM before the next
    bookkeeping launch; the three runs dispatch the same sequence, so the counter files are matched to
    the trace by position."""
    def dispatches(path, counter=None):
        rows = []
        with open(path) as f:
            for r in csv.DictReader(f):
                if counter and r["Counter_Name"] != counter:
                    continue
                rows.append(r)
        rows.sort(key=lambda r: int(r["Dispatch_Id"]))
        return rows
    trace = dispatches(trace_csv)
    fetch, write = dispatches(fetch_csv, "FETCH_SIZE"), dispatches(write_csv, "WRITE_SIZE")
    if not (len(trace) == len(fetch) == len(write)):
        sys.exit(f"dispatch counts differ: trace {len(trace)}, fetch {len(fetch)}, write {len(write)}")
    copy = [i for i, r in enumerate(trace) if short(r["Kernel_Name"]).startswith("stream_copy_kernel")]
    f_scale = (COPY_BYTES / 1024.0) / (sum(float(fetch[i]["Counter_Value"]) for i in copy) / len(copy))
    w_scale = (COPY_BYTES / 1024.0) / (sum(float(write[i]["Counter_Value"]) for i in copy) / len(copy))
    step_kernels = ("decode_meta_norm_kernel", "gemm_mfma_kernel", "gemv_mfma_kernel", "wgemm_kernel",
                    "splitk_reduce", "decode_attn", "rmsnorm")
    steps = collections.defaultdict(list)             # batch -> list of steps (lists of dispatch indices)
    cur = None
    for i, r in enumerate(trace):
        name = short(r["Kernel_Name"])
        if name.startswith("decode_meta_norm_kernel"):
            cur = [i]
            steps[int(r["Grid_Size_X"]) // int(r["Workgroup_Size_X"]) - 1].append(cur)
        elif cur is not None and name.startswith(step_kernels):
            cur.append(i)
        else:
            cur = None
    gemm_names = ["QKV projection", "O projection + residual", "gate/up + SwiGLU", "down projection + residual"]
    print("| batch | launch | kernel | workgroups x K splits | threads | mean us | fetched MB | written MB |")
    print("|---|---|---|---|---|---|---|---|")
    for B in sorted(steps):
        runs = [s for s in steps[B] if len(s) == len(steps[B][-1])]
        total = 0.0
        n_gemm = 0
        for pos in range(len(runs[0])):
            idx = [s[pos] for s in runs]
            r = trace[idx[0]]
            name = short(r["Kernel_Name"])
            us = sum((int(trace[i]["End_Timestamp"]) - int(trace[i]["Start_Timestamp"])) / 1e3 for i in idx) / len(idx)
            fm = sum(float(fetch[i]["Counter_Value"]) for i in idx) / len(idx) * f_scale * 1024 / 1e6
            wm = sum(float(write[i]["Counter_Value"]) for i in idx) / len(idx) * w_scale * 1024 / 1e6
            what = ""
            if name.startswith(("gemm_mfma_kernel", "gemv_mfma_kernel", "wgemm_kernel")):
                what = gemm_names[n_gemm] if n_gemm < 4 else ""
                n_gemm += 1
            elif name.startswith("splitk_reduce"):
                what = "sum of the K splits"
            wgx = int(r["Grid_Size_X"]) // int(r["Workgroup_Size_X"])
            print(f"| {B} | {what} | `{name}` | {wgx} x {r['Grid_Size_Y']} | {r['Workgroup_Size_X']} | {us:.1f} | {fm:.1f} | {wm:.1f} |")
            total += us
        print(f"| {B} | all launches of the step | | | | {total:.1f} | | |")


def summarise(fetch_csv, write_csv):
    fetch, write = read_counter(fetch_csv, "FETCH_SIZE"), read_counter(write_csv, "WRITE_SIZE")
    mean = lambda v: sum(v) / len(v)
    copy_key = next(k for k in fetch if k[0].startswith("stream_copy_kernel"))
    known_kib = COPY_BYTES / 1024.0
    f_scale = known_kib / mean(fetch[copy_key])
    w_scale = known_kib / mean(write[copy_key])
    print(f"copy kernel: {known_kib:.0f} KiB each way; FETCH_SIZE reads {mean(fetch[copy_key]):.0f}, "
          f"WRITE_SIZE reads {mean(write[copy_key]):.0f} -> scale factors {f_scale:.4f} (fetch), {w_scale:.4f} (write)")
    print()
    print("| kernel | grid (threads) | dispatches | fetched MB | written MB | total MB |")
    print("|---|---|---|---|---|---|")
    for key in sorted(fetch, key=lambda k: -mean(fetch[k])):
        if key not in write:
            continue
        fm = mean(fetch[key]) * f_scale * 1024 / 1e6
        wm = mean(write[key]) * w_scale * 1024 / 1e6
        if fm + wm < 1.0:
            continue
        print(f"| `{key[0]}` | {key[1]} | {len(fetch[key])} | {fm:.1f} | {wm:.1f} | {fm + wm:.1f} |")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--summarise", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"))
    ap.add_argument("--durations", metavar="KERNEL_TRACE_CSV")
    ap.add_argument("--decode-steps", nargs=3, metavar=("KERNEL_TRACE_CSV", "FETCH_CSV", "WRITE_CSV"))
    ap.add_argument("--decode-batches", default="", help="comma-separated decode batches instead of prefill + batch 256")
    args = ap.parse_args()
    if args.summarise:
        summarise(*args.summarise)
    elif args.durations:
        durations(args.durations)
    elif args.decode_steps:
        decode_steps(*args.decode_steps)
    else:
        workload([int(b) for b in args.decode_batches.split(",")] if args.decode_batches else None)


if __name__ == "__main__":
    main()
