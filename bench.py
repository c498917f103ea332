#!/usr/bin/env python3
"""Benchmark of the S2-Attn hot path (forward + backward) on one MI355X.

One step = one forward and one backward pass of a whole S2-Attn layer over one batch of
synthetic inputs (iid N(0,1), rounded to bf16) that are resident in HBM before the timed
region.  The default workload is the Llama2-7B-shaped layer at N = 32768, G = 8192.
Prints ONE JSON line: effective TFLOP/s (only in-group causal pairs are counted:
14*D FLOP per (query, key) pair for forward + backward), the roofline of the dominant
kernel measured with HIP events on the launch stream, and the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
CSRC = os.path.join(ROOT, "paper_2309_12307_amd", "csrc")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def source_hash() -> str:
    """sha256 over the kernel sources, to tie profiled figures to the code they were measured on."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        if name.endswith((".hip", ".h")) and name != "s2attn_probes.hip":
            h.update(name.encode())
            h.update(open(os.path.join(CSRC, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, algo: str, kernel: str):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
    recorded in profiles/hbm_traffic.txt (not measurable from inside the process).  None when
    the workload was not profiled or the kernel sources have changed since."""
    if not os.path.exists(TRAFFIC_FILE):
        return None
    recorded_hash, table = None, {}
    for line in open(TRAFFIC_FILE):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "source_sha256":
            recorded_hash = f[1]
        elif len(f) == 4:
            table[(f[0], f[1], f[2])] = float(f[3])
    if recorded_hash != source_hash():
        return None
    return table.get((workload, algo, kernel))


class HipEvents:
    """Raw HIP events through the runtime torch already loaded, so they can be
    recorded on the stream the library launches on."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self) -> int:
        e = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(e))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        return e.value

    def record(self, ev: int, stream: int) -> None:
        rc = self.hip.hipEventRecord(ev, stream)
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def destroy(self, ev: int) -> None:
        self.hip.hipEventDestroy(ev)


def cpu_baseline(cfg, inp, budget_s=15.0):
    """The oracle as it stands, on a bounded sample: whole (kv head, group) slices of the
    workload, forward + backward in fp32, until about `budget_s` seconds are spent."""
    from oracle import s2attn_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    r = cfg.H // cfg.Hkv
    pairs_per_slice = r * cfg.G * (cfg.G + 1) // 2
    picks = [(c, g) for g in range(cfg.N // cfg.G) for c in range(cfg.Hkv)]
    done, t_total = 0, 0.0
    for c, g in picks:
        t0 = time.perf_counter()
        orc.s2attn_group_slice(inp["q"], inp["k"], inp["v"], inp["do"], cfg.G, 0, c, g, dtype=np.float32)
        t_total += time.perf_counter() - t0
        done += 1
        if t_total > budget_s:
            break
    flops = 14.0 * cfg.D * pairs_per_slice * done
    return {
        "value": flops / t_total / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
        "sample": f"{done} of {cfg.B * cfg.Hkv * (cfg.N // cfg.G)} (kv head, group) slices of {cfg.name}, "
                  f"fwd+bwd in fp32 numpy, {t_total:.1f} s",
    }


def run_probes():
    path = os.path.join(ROOT, "paper_2309_12307_amd", "libs2attn_probes.so")
    if not os.path.exists(path):
        raise SystemExit(f"{path} not found: build it with `python -m paper_2309_12307_amd.build`")
    L = ctypes.CDLL(path)
    dbl = ctypes.c_double
    out = {"probe": "MI355X bf16 32x32x16 MFMA rate against operand data, L2 fp32 atomic rate",
           "unit": "TFLOP/s", "mfma_registers": {}, "mfma_lds_operand": []}

    def call(f, *a):
        v = dbl()
        rc = f(*a, ctypes.byref(v))
        if rc != 0:
            raise RuntimeError(f"probe failed with hipError {rc}")
        return v.value

    for mode, name in ((0, "ones"), (1, "randn")):
        out["mfma_registers"][name] = round(call(L.s2probe_mfma_registers, mode), 1)
    work = {0: "none", 1: "3 fma + 1 exp2 per MFMA", 2: "4 fma + 2 exp2 per MFMA"}
    for waves in (2, 1):
        for tr in (0, 1):
            for vw in (0, 1, 2):
                for reuse in (1, 2):
                    row = {"waves_per_simd": waves, "fragments": "transposed 2 x b64" if tr else "row-major b128",
                           "vector_work": work[vw], "mfma_per_lds_fragment": reuse}
                    for mode, name in ((0, "ones"), (1, "randn")):
                        row[name] = round(call(L.s2probe_mfma_lds, tr, vw, waves, reuse, mode), 1)
                    out["mfma_lds_operand"].append(row)
                    print(row, file=sys.stderr, flush=True)
    out["l2_fp32_atomic_add_TB_per_s"] = round(call(L.s2probe_atomic_add), 3)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 20; 100 for C2, whose step is under a millisecond)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed steps before them (default 10, about 90 ms of C3: after an idle period the chip "
                         "takes about 45 ms of load to reach its steady clock; 60 for C2)")
    ap.add_argument("--workload", default="C3",
                    help="C2 | C3 | C4 | C5 (bf16 configurations); a '-full' suffix (e.g. C3-full) runs plain "
                         "full causal attention of the same layer through the same kernels (G = N, no head "
                         "shifts), for the S2-Attn : full attention time ratio")
    ap.add_argument("--bwd-algo", choices=["auto", "recompute", "stored"], default="auto",
                    help="how the backward's dQ kernel gets dS: recomputed (what 'auto' picks) or stored by the "
                         "dK/dV kernel in the workspace (2 bytes per (query, key) pair)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--operands", choices=["normal", "zero"], default="normal",
                    help="'zero' runs the same launches on all-zero q, k, v, dO: not the workload (the line says so "
                         "in 'data'), a probe of how much of the time is the chip's data-dependent power limit")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy, so that a rocprofv3 --pmc run of this "
                         "command holds a kernel of known HBM traffic to scale FETCH_SIZE/WRITE_SIZE by")
    ap.add_argument("--probes", action="store_true",
                    help="instead of the benchmark, run the hardware probes of libs2attn_probes.so (bf16 MFMA rate "
                         "against operand data, with register and LDS operands and softmax-like vector work; L2 "
                         "fp32 atomic-add rate) and print them as one JSON line")
    ap.add_argument("--source-hash", action="store_true", help="print the hash of the kernel sources and exit")
    args = ap.parse_args()
    if args.source_hash:
        print(source_hash())
        return
    if args.probes:
        run_probes()
        return
    short_step = args.workload.startswith("C2")
    if args.steps is None:
        args.steps = 100 if short_step else 20
    if args.warmup is None:
        args.warmup = 60 if short_step else 10
    if args.gpus != 1:
        print("bench.py measures the single-GPU S2-Attn kernels only: this build has no multi-GPU path "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2309_12307_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback)", file=sys.stderr)
        sys.exit(2)
    full = args.workload.endswith("-full")
    cfg = inputs.CONFIGS[args.workload[:-5] if full else args.workload]
    if full:
        cfg = inputs.S2Config(cfg.name + "-full", cfg.index, cfg.dtype, cfg.B, cfg.N, cfg.H, cfg.Hkv, cfg.D, cfg.N)
    rule = binding.SHIFT_NONE if full else binding.SHIFT_SECOND_HALF
    if cfg.dtype != "bf16":
        raise SystemExit("bench workloads are the bf16 configurations")
    binding.lib()   # fail loudly before any work if the library is missing

    inp = inputs.make_config_inputs(cfg)

    def dev(name):
        return torch.from_numpy(inp[name + "_bits"].view(np.int16)).cuda().view(torch.bfloat16)

    q, k, v, do = dev("q"), dev("k"), dev("v"), dev("do")
    if args.operands == "zero":
        for t in (q, k, v, do):
            t.zero_()
    o = torch.empty_like(q)
    lse = torch.empty((cfg.B, cfg.H, cfg.N), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    algo = {"auto": binding.BWD_AUTO, "recompute": binding.BWD_RECOMPUTE, "stored": binding.BWD_STORED_DS}[args.bwd_algo]
    p_fwd = binding.make_params(q, k, v, o, lse, cfg.G, shift_rule=rule)
    p_bwd = binding.make_params(q, k, v, o, lse, cfg.G, dout=do, dq=dq, dk=dk, dv=dv, shift_rule=rule, bwd_algo=algo)
    ws = torch.empty(binding.bwd_workspace_bytes_ex(p_bwd), dtype=torch.uint8, device="cuda")
    p_bwd = binding.make_params(q, k, v, o, lse, cfg.G, dout=do, dq=dq, dk=dk, dv=dv, workspace=ws, shift_rule=rule,
                                bwd_algo=algo)
    stream = torch.cuda.current_stream().cuda_stream
    ev = HipEvents()

    def step(marks=None):
        if marks is not None:
            ev.record(marks[0], stream)
        binding.s2attn_fwd_ex(p_fwd, stream=stream)
        if marks is not None:
            binding.s2attn_bwd_ex_marked(p_bwd, marks[1:5], stream=stream)
        else:
            binding.s2attn_bwd_ex(p_bwd, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    marks = [[ev.create() for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(marks[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-kernel durations from the events of the timed region
    names = ["fwd", "bwd_delta", "bwd_dkdv", "bwd_dq"]
    dur = {n: 0.0 for n in names}
    for m in marks:
        for j, n in enumerate(names):
            dur[n] += ev.elapsed_ms(m[j], m[j + 1])
    for n in names:
        dur[n] /= args.steps
    # per-step device times from the same events: forward alone, backward alone (with the
    # delta pre-pass) and both
    per_step = {"fwd": [ev.elapsed_ms(m[0], m[1]) for m in marks],
                "bwd": [ev.elapsed_ms(m[1], m[4]) for m in marks],
                "fwd_bwd": [ev.elapsed_ms(m[0], m[4]) for m in marks]}
    spread = {k_: {"median_ms": float(np.median(v_)), "min_ms": float(np.min(v_))} for k_, v_ in per_step.items()}
    for m in marks:
        for e in m:
            ev.destroy(e)

    pairs = cfg.B * cfg.H * cfg.N * (cfg.G + 1) / 2.0
    flops_total = binding.effective_flops(cfg.B, cfg.N, cfg.H, cfg.D, cfg.G, 2)
    # algorithmic FLOPs per launch: forward 4D per pair; dK/dV kernel 8D (S, dP, dV, dK);
    # dQ kernel 2D (its recomputation of S and dP is not credited)
    alg = {"fwd": 4.0 * cfg.D * pairs, "bwd_dkdv": 8.0 * cfg.D * pairs, "bwd_dq": 2.0 * cfg.D * pairs}
    kernels = {n: {"ms": dur[n], "algorithmic_tflops": alg[n] / dur[n] / 1e9 if n in alg else None} for n in names}
    dom = max(alg, key=lambda n: dur[n])
    achieved = alg[dom] / dur[dom] / 1e9
    traffic = measured_traffic(cfg.name, "stored" if args.bwd_algo == "stored" else "recompute", dom)

    value = flops_total / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": "S2-Attn fwd+bwd effective TFLOP/s (in-group causal FLOPs only)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic" if args.operands == "normal" else "all-zero operands (power probe)",
        "config": {"workload": f"{cfg.name}: S2-Attn layer fwd+bwd, B={cfg.B} N={cfg.N} H={cfg.H} Hkv={cfg.Hkv} "
                               f"D={cfg.D} G={cfg.G} " +
                               ("no head shifts (full causal attention)" if full
                                else f"shift={cfg.G // 2} on heads >= H/2"),
                   "effective_tflop_per_step": flops_total / 1e12,
                   "backward": "dS stored by the dK/dV kernel, read back by the dQ kernel" if args.bwd_algo == "stored"
                               else "dS recomputed in the dQ kernel",
                   "workspace_bytes": int(ws.numel())},
        "frac_of_bf16_mfma_peak": value / PEAK_BF16_TFLOPS,
        "device_time_per_step": spread,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic},
        "kernels": kernels,
    }
    # (one full-attention slice would be the whole N x N problem; the zero probe is not the workload)
    if not args.no_cpu_baseline and not full and args.operands == "normal":
        out["cpu_baseline"] = cpu_baseline(cfg, inp)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
