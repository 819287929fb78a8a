"""HBM-traffic probe: launches the benchmark's dominant kernels a few times, each at the shape the
benchmark runs it, plus a plain device copy of known size, so that one `rocprofv3 --pmc` pass per
counter gives bytes per launch and the copy gives the counter's scale.

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT/fetch -- python3 -m paper_2107_06469_amd.traffic_probe
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT/write -- python3 -m paper_2107_06469_amd.traffic_probe
    python3 -m paper_2107_06469_amd.traffic_probe --summarise OUT/fetch OUT/write
    rocprofv3 --pmc GRBM_GUI_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 --output-format csv -d OUT/mfma \
        -- python3 -m paper_2107_06469_amd.traffic_probe
    python3 -m paper_2107_06469_amd.traffic_probe --mfma OUT/mfma

Shapes are workload 1's (8 models, 4096 x 4096 layers, batch 512, bf16 with fp32 Adam state).
The summary prints, per kernel, the mean counter value per launch (KiB), the copy's reading and the
factor that turns counter KiB into bytes (known copy bytes / copy reading), and the scaled bytes.
"""
from __future__ import annotations

import argparse
import csv
import glob
import os
import sys
from collections import defaultdict

COPY_BYTES = 1 << 30      # bytes read (and as many written) by the reference copy
REPS = 3


def run():
    import torch
    from . import ops
    G, d, B = 8, 4096, 512
    bf = torch.bfloat16
    n = d * d
    dz = [torch.randn(B, d, device="cuda").to(bf) for _ in range(G)]
    h = [torch.randn(B, d, device="cuda").to(bf) for _ in range(G)]
    p = [torch.randn(n, device="cuda") for _ in range(G)]
    m = [torch.zeros(n, device="cuda") for _ in range(G)]
    v = [torch.zeros(n, device="cuda") for _ in range(G)]
    w16 = [t.to(bf) for t in p]
    g = [torch.zeros(n, device="cuda") for _ in range(G)]
    out = [torch.zeros(B, d, dtype=bf, device="cuda") for _ in range(G)]
    pre = [torch.zeros(B, d, dtype=bf, device="cuda") for _ in range(G)]
    bias = [torch.zeros(d, device="cuda") for _ in range(G)]
    hp = [(1e-3, 0.9, 0.999, 1e-8, 10.0, 1000.0)] * G
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
    dst = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for _ in range(REPS):
        # weight gradient + Adam in the epilogue: dW[d, d] = dz^T h
        ops.hydra_op_gemm_update(ops.BF16, d, d, B, dz, h, 1, p, m, v, w16, hp, ldx=d, ldw=d, ldo=d)
        # forward Linear + GeLU, input gradient with GeLU', plain weight gradient, Adam over one layer
        ops.hydra_op_gemm(ops.BF16, B, d, d, h, w16, out, x_kmajor=True, w_kmajor=True, ldx=d, ldw=d, ldo=d,
                          bias=bias, pre=pre, act=ops.EPI_GELU)
        ops.hydra_op_gemm(ops.BF16, B, d, d, dz, w16, out, x_kmajor=True, w_kmajor=False, ldx=d, ldw=d, ldo=d,
                          gate=pre, ldg=d, act=ops.EPI_GELU)
        ops.hydra_op_gemm(ops.BF16, d, d, B, dz, h, g, x_kmajor=False, w_kmajor=False, ldx=d, ldw=d, ldo=d, out_f32=True)
        ops.hydra_op_optim(1, n, p, g, m, v, w16, hp)
        dst.copy_(src)
        torch.cuda.synchronize()
    print("traffic_probe: done", flush=True)


def _read(dirname):
    """kernel name -> list of counter values (one per dispatch), from rocprofv3's counter_collection csv"""
    rows = defaultdict(list)
    for path in glob.glob(os.path.join(dirname, "**", "*counter_collection.csv"), recursive=True):
        with open(path, newline="") as f:
            for r in csv.DictReader(f):
                rows[(r["Kernel_Name"], r["Counter_Name"])].append(float(r["Counter_Value"]))
    return rows


def _label(kernel: str) -> str:
    from .profile_summary import short
    return short(kernel)


def summarise(fetch_dir, write_dir):
    out = {}
    for counter, dirname in (("FETCH_SIZE", fetch_dir), ("WRITE_SIZE", write_dir)):
        rows = _read(dirname)
        copy = [(k, v) for (k, c), v in rows.items() if c == counter and ("copy" in k.lower() or "elementwise" in k.lower())
                and abs(max(v)) > 0]
        # the reference copy is the dispatch with the largest reading among the copy/elementwise kernels
        ck, cv = max(copy, key=lambda kv: max(kv[1]))
        factor = COPY_BYTES / (max(cv) * 1024.0)
        print(f"{counter}: copy of {COPY_BYTES} bytes reads {max(cv):.0f} KiB -> factor {factor:.4f} (bytes per counter KiB / 1024)")
        for (k, c), v in sorted(rows.items()):
            if c != counter or "hydra" not in k:
                continue
            mean = sum(v) / len(v)
            out.setdefault(_label(k), {})[counter] = mean * 1024.0 * factor
            print(f"  {_label(k):90s} launches {len(v):3d}  mean {mean:12.0f} KiB  scaled {mean * 1024.0 * factor / 1e6:10.1f} MB")
    print("per launch, fetch + write (MB):")
    for k, d in out.items():
        print(f"  {k:90s} {sum(d.values()) / 1e6:10.1f}")


N_SIMD = 256 * 4          # SIMDs of the chip; one issues 1024 bf16 MFMA flops per clock
N_XCD = 8                 # GRBM_GUI_ACTIVE comes back summed over the 8 XCDs' counters


def mfma(dirname):
    """Matrix-core occupancy from hardware counters: busy cycles of the MFMA pipes over the clock cycles the
    kernel was active (the chip's own clock, whatever it ran at), the flops the counters saw, and the clock
    itself (active cycles / dispatch duration)."""
    per = defaultdict(lambda: defaultdict(list))
    for path in glob.glob(os.path.join(dirname, "**", "*counter_collection.csv"), recursive=True):
        with open(path, newline="") as f:
            for r in csv.DictReader(f):
                if "hydra" not in r["Kernel_Name"]:
                    continue
                d = per[_label(r["Kernel_Name"])]
                d[r["Counter_Name"]].append(float(r["Counter_Value"]))
                if r["Counter_Name"] == "GRBM_GUI_ACTIVE":
                    d["ns"].append(float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
    print(f"{'kernel':72s} {'us':>8s} {'clock GHz':>9s} {'MFMA busy %':>11s} {'TFLOP (counter)':>15s} {'TFLOP/s':>8s} {'of 2.5 PF':>9s}")
    for k, d in sorted(per.items()):
        mean = {c: sum(v) / len(v) for c, v in d.items()}
        if not all(c in mean for c in ("GRBM_GUI_ACTIVE", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "ns")):
            continue
        act, busy, fl = mean["GRBM_GUI_ACTIVE"] / N_XCD, mean["SQ_VALU_MFMA_BUSY_CYCLES"], mean["SQ_INSTS_VALU_MFMA_MOPS_BF16"] * 512
        rate = fl / (mean["ns"] * 1e-9) / 1e12
        print(f"{k[:72]:72s} {mean['ns'] / 1e3:8.1f} {act / mean['ns']:9.2f} {100 * busy / (act * N_SIMD):11.1f} "
              f"{fl / 1e12:15.4f} {rate:8.0f} {rate / 2500:9.3f}")


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--summarise", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"))
    ap.add_argument("--mfma", metavar="DIR")
    a = ap.parse_args()
    if a.summarise:
        summarise(*a.summarise)
    elif a.mfma:
        mfma(a.mfma)
    else:
        run()
    sys.exit(0)
