#!/usr/bin/env python3
"""Benchmark of the fused decoder-block forward on one MI355X.

One "step" is one whole forward of the workload: embedding -> L fused decoder
layers (norm, QKV GEMM, fused causal attention, out GEMM + residual, norm, MLP
GEMMs with fused activation / residual) -> final norm -> tied LM head, on
synthetic seeded inputs that are resident in HBM before the timed region.

Default workload: the 12-layer GPT-2-small-shaped model, bf16, batch 8 x 1024
tokens.  Prints ONE JSON line with the whole-job throughput in tokens/s, the
roofline of the dominant kernel (measured with HIP events on the launch stream)
and the fp64 CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="stop adding oracle samples once this much CPU time is spent")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="launch a plain copy of known size, then the per-launch GEMM loop of the roofline "
                         "section, and exit: the program to run under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE`")
    ap.add_argument("--traffic-summarize", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="turn the two counter_collection.csv files of the probe runs into "
                         "profiles/hbm_traffic.json (no GPU needed)")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------
# HBM traffic of the dominant kernel from hardware counters (collected offline, see --traffic-probe)
# ---------------------------------------------------------------------------------------------

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_SOURCES = ["gemm_bf16.hip", "common.hpp"]
COPY_BYTES = 256 << 20          # the probe's copy kernel reads and writes this many bytes


def kernel_source_digest():
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2604_16498_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def recorded_traffic(workload, kernel):
    """Bytes per launch measured for `kernel` on `workload`, or None when there is no record or
    the kernel sources have changed since the counters were taken."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    if rec.get("source_sha256") != kernel_source_digest() or rec.get("workload") != workload:
        return None
    # "gemm_bf16_pers<128,128,2,2> act=none" -> template instantiation "<128,128,2,2,ACT,MODE>"
    variant, _, act = kernel.partition(" act=")
    from paper_2604_16498_amd import binding as F
    inst = "%s,%d,0>" % (variant[:-1], F.ACT.get(act, 0))
    ent = rec.get("kernels", {}).get(inst)
    return None if ent is None else round(ent["fetch_bytes_per_launch"] + ent["write_bytes_per_launch"])


def summarize_traffic(fetch_csv, write_csv):
    """FETCH_SIZE / WRITE_SIZE are reported in KiB per dispatch; both are scaled by what the same
    counter reads for the copy kernel of COPY_BYTES (read once, written once)."""
    import csv
    import re

    def per_kernel(path, counter):
        acc = {}
        with open(path) as f:
            for r in csv.DictReader(f):
                if r["Counter_Name"] != counter:
                    continue
                acc.setdefault((r["Kernel_Name"], r["Dispatch_Id"]), 0.0)
                acc[(r["Kernel_Name"], r["Dispatch_Id"])] += float(r["Counter_Value"])
        out = {}
        for (name, _), v in acc.items():
            out.setdefault(name, []).append(v)
        return out

    def short(name):
        m = re.search(r"(gemm_bf16_\w+?)_kernel<([^>]*)>", name)
        return "%s<%s>" % (m.group(1), m.group(2).replace(" ", "")) if m else name[:60]

    fetch, write = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    copy = [k for k in fetch if "copy" in k.lower()]
    if not copy:
        raise SystemExit("no copy kernel found in %s" % fetch_csv)
    ck = max(copy, key=lambda k: max(fetch[k]))
    # skip the first launch of every kernel (cold caches, first-touch)
    mean = lambda v: sum(v[1:]) / max(1, len(v) - 1) if len(v) > 1 else v[0]
    # the runtime's copy kernel also serves small transfers: keep the probe's large copies only
    big = lambda v: [x for x in v if x > 0.5 * max(v)]
    f_scale = COPY_BYTES / (mean(big(fetch[ck])) * 1024.0)
    w_scale = COPY_BYTES / (mean(big(write[ck])) * 1024.0)
    kernels = {}
    for k in fetch:
        if "gemm_bf16" not in k:
            continue
        kernels[short(k)] = {
            "launches": len(fetch[k]),
            "fetch_bytes_per_launch": mean(fetch[k]) * 1024.0 * f_scale,
            "write_bytes_per_launch": mean(write.get(k, [0.0])) * 1024.0 * w_scale,
        }
    rec = {"workload": None, "source_sha256": kernel_source_digest(), "copy_kernel": ck[:80],
           "copy_bytes": COPY_BYTES, "fetch_scale": f_scale, "write_scale": w_scale, "kernels": kernels}
    return rec



# ---------------------------------------------------------------------------------------------
# model construction (device memory plumbing only)
# ---------------------------------------------------------------------------------------------

def build_model(wl, F, torch, I):
    """Weights, descriptors, caches, workspace and the input of one workload on the GPU."""
    sh = wl.block
    dt = torch.bfloat16 if wl.bf16 else torch.float32
    big = sh.d_model >= 4096          # 8B-shaped: draw on the device (host generation takes minutes)
    g = torch.Generator(device="cuda").manual_seed(I.BASE_SEED * 1000 + wl.cid)

    def dev(a):
        if a is None:
            return None
        t = torch.from_numpy(a)
        return (t.to(torch.bfloat16) if wl.bf16 else t).cuda()

    def dev_normal(shape, std):
        return (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * std).to(dt)

    layers = []
    for l in range(wl.layers):
        if not big:
            w = {k: dev(v) for k, v in I.block_weights(sh, wl.cid, l, wl.bf16, wl.bias_std).items()}
        else:
            d = sh.d_model
            w = {
                "norm1_g": torch.ones(d, device="cuda", dtype=dt), "norm1_b": None,
                "w_qkv": dev_normal((sh.qkv_out, d), 0.02), "b_qkv": None,
                "w_o": dev_normal((d, sh.q_heads * sh.head_dim), 0.02), "b_o": None,
                "norm2_g": torch.ones(d, device="cuda", dtype=dt), "norm2_b": None,
                "w_up": dev_normal((sh.up_out, d), 0.02), "b_up": None,
                "w_down": dev_normal((d, sh.d_ff), 0.02), "b_down": None,
            }
        layers.append(w)
    mw = {k: dev(v) for k, v in I.model_weights(wl).items()}
    descs = [F.make_block_desc(sh, w) for w in layers]
    # logits rows padded to a multiple of 8 elements (16-byte aligned rows, the usual vocabulary
    # padding); the padding columns are never written or read
    logits_ld = (wl.vocab + 7) // 8 * 8
    model = F.make_model_desc(descs, mw, logits_ld=logits_ld)

    B, S = wl.batch, wl.seq
    cap = wl.pos0 + S
    cap = (cap + 63) // 64 * 64
    kshape = (wl.layers, B, sh.kv_heads, cap, sh.head_dim)
    if wl.pos0:
        kc = torch.randn(kshape, generator=g, device="cuda", dtype=torch.float32).to(dt)
        vc = torch.randn(kshape, generator=g, device="cuda", dtype=torch.float32).to(dt)
    else:
        kc = torch.zeros(kshape, device="cuda", dtype=dt)
        vc = torch.zeros_like(kc)
    if wl.vocab:
        ids_host = I.token_ids(wl.cid, B, S, wl.vocab)
        inp = torch.from_numpy(ids_host).cuda()
        out = torch.empty(B, S, logits_ld, device="cuda", dtype=dt)
    else:
        ids_host = None
        inp = dev(I.hidden_states(wl))
        out = torch.empty(B, S, sh.d_model, device="cuda", dtype=dt)
    ws = F.workspace(F.forge_model_workspace_bytes(model, B, S, cap))
    keep = (layers, mw, descs)
    return dict(model=model, inp=inp, out=out, kc=kc, vc=vc, ws=ws, keep=keep, ids_host=ids_host,
                layers=layers, mw=mw, cap=cap, logits_ld=logits_ld)


# ---------------------------------------------------------------------------------------------
# algorithmic work
# ---------------------------------------------------------------------------------------------

def gemm_launches(wl):
    """The plain (non head-split) GEMM launches of one step: (name, M, N_out, K, act, count)."""
    sh = wl.block
    T = wl.batch * wl.seq
    hd = sh.q_heads * sh.head_dim
    out = [
        ("out", T, sh.d_model, hd, "none", wl.layers),
        ("mlp_up", T, sh.d_ff, sh.d_model, sh.mlp_act, wl.layers),
        ("mlp_down", T, sh.d_model, sh.d_ff, "none", wl.layers),
    ]
    if wl.vocab:
        out.append(("lm_head", T, wl.vocab, sh.d_model, "none", 1))
    return out


def step_flops(wl):
    sh = wl.block
    T = wl.batch * wl.seq
    hd = sh.q_heads * sh.head_dim
    kv = wl.pos0 + wl.seq
    gemm = 2.0 * T * (sh.qkv_out * sh.d_model + sh.d_model * hd + sh.up_out * sh.d_model
                      + sh.d_model * sh.d_ff) * wl.layers
    if wl.vocab:
        gemm += 2.0 * T * wl.vocab * sh.d_model
    # causal attention: only the keys a query may see (lower triangle incl. diagonal)
    pairs = wl.batch * sum(wl.pos0 + s + 1 for s in range(wl.seq)) if wl.seq <= 8192 else 0
    attn = 4.0 * sh.q_heads * sh.head_dim * pairs * wl.layers
    return gemm, attn


def step_bytes(wl):
    """Algorithmic HBM bytes of one step for the bandwidth-bound (decode) workload: every weight
    and every cached K/V row is read once."""
    sh = wl.block
    es = 2 if wl.bf16 else 4
    hd = sh.q_heads * sh.head_dim
    wbytes = (sh.qkv_out * sh.d_model + sh.d_model * hd + sh.up_out * sh.d_model + sh.d_model * sh.d_ff) * es
    kvbytes = 2 * wl.batch * sh.kv_heads * (wl.pos0 + wl.seq) * sh.head_dim * es
    return (wbytes + kvbytes) * wl.layers


# ---------------------------------------------------------------------------------------------

def main():
    args = parse()
    if args.traffic_summarize:
        from paper_2604_16498_amd import inputs as I
        rec = summarize_traffic(*args.traffic_summarize)
        rec["workload"] = I.WORKLOADS[int(args.workload[1])].name
        with open(TRAFFIC_FILE, "w") as f:
            json.dump(rec, f, indent=1)
        print(json.dumps(rec, indent=1))
        return
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_16498_amd import binding as F
    from paper_2604_16498_amd import inputs as I
    F.lib()                                    # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    wl = I.WORKLOADS[int(args.workload[1])]
    m = build_model(wl, F, torch, I)
    pos0 = wl.pos0
    if args.traffic_probe:
        src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()

    def step():
        F.forge_model_forward(m["model"], m["inp"], m["out"], m["kc"], m["vc"], pos0, m["ws"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(1 if args.traffic_probe else args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / (1 if args.traffic_probe else args.steps)
    tokens = wl.batch * wl.seq
    value = tokens / (ms_per_step * 1e-3)
    gemm_fl, attn_fl = step_flops(wl)

    # ---- per-step latency distribution (outside the timed region): HIP events around single steps
    latency = None
    if not args.traffic_probe:
        evs = []
        for _ in range(50):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            step()
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ds = sorted(a.elapsed_time(b) for a, b in evs)
        latency = {"steps": len(ds), "mean": round(sum(ds) / len(ds), 4), "p50": round(ds[len(ds) // 2], 4),
                   "p90": round(ds[int(len(ds) * 0.9)], 4), "p99": round(ds[min(len(ds) - 1, int(len(ds) * 0.99))], 4)}

    # ---- the same step through the compiled executor (static buffer plan + HIP graph replay),
    # outside the timed region: reported beside the plain launch list, never as `value`
    compiled = None
    if not args.traffic_probe:
        cm = F.CompiledModel(m["model"], wl.batch, wl.seq, pos0, m["cap"])
        cws = F.workspace(cm.workspace_bytes())
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        cm.bind(m["inp"], m["out"], m["kc"], m["vc"], cws, side)
        for _ in range(args.warmup):
            cm.run(side)
        side.synchronize()
        c0 = time.perf_counter()
        for _ in range(args.steps):
            cm.run(side)
        side.synchronize()
        c_ms = (time.perf_counter() - c0) * 1e3 / args.steps
        evs = []
        with torch.cuda.stream(side):
            for _ in range(50):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                cm.run(side)
                e1.record()
                evs.append((e0, e1))
        side.synchronize()
        ds = sorted(a.elapsed_time(b) for a, b in evs)
        # host time to enqueue one step (the calls return before the GPU is done)
        torch.cuda.synchronize()
        h0 = time.perf_counter()
        for _ in range(10):
            step()
        h_plain = (time.perf_counter() - h0) / 10
        torch.cuda.synchronize()
        h0 = time.perf_counter()
        for _ in range(10):
            cm.run(side)
        h_comp = (time.perf_counter() - h0) / 10
        side.synchronize()
        ni, nr, _, nb = cm.counts()
        compiled = {"ms_per_step": round(c_ms, 4), "p50": round(ds[len(ds) // 2], 4),
                    "host_enqueue_us": round(h_comp * 1e6, 1), "plain_host_enqueue_us": round(h_plain * 1e6, 1),
                    "p99": round(ds[min(len(ds) - 1, int(len(ds) * 0.99))], 4),
                    "instructions": ni, "registers": nr, "buffers": nb, "rho_buf": round(1 - nb / nr, 3),
                    "workspace_bytes": cm.workspace_bytes(), "plain_workspace_bytes": m["ws"].numel()}
        cm.close()
        del cws
        torch.cuda.synchronize()

    # ---- the decode step on int8 weights (quantised here by the library's own kernel), outside
    # the timed region: reported beside the bf16 step, never as `value`
    w8 = None
    if args.workload == "c5" and not args.traffic_probe:
        layers8 = []
        for w in m["layers"]:
            d = dict(w)
            for wn, sn in (("w_qkv", "s_qkv"), ("w_o", "s_o"), ("w_up", "s_up"), ("w_down", "s_down")):
                d[wn], d[sn] = F.forge_quantize_int8(w[wn])
            layers8.append(d)
        descs8 = [F.make_block_desc(wl.block, d) for d in layers8]
        model8 = F.make_model_desc(descs8, m["mw"], logits_ld=m["logits_ld"])
        ws8 = F.workspace(F.forge_model_workspace_bytes(model8, wl.batch, wl.seq, m["cap"]))

        def step8():
            F.forge_model_forward(model8, m["inp"], m["out"], m["kc"], m["vc"], pos0, ws8)

        for _ in range(args.warmup):
            step8()
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(args.steps):
            step8()
        torch.cuda.synchronize()
        ms8 = (time.perf_counter() - c0) * 1e3 / args.steps
        shb = wl.block
        wbytes8 = (shb.qkv_out * shb.d_model + shb.d_model * shb.q_heads * shb.head_dim + shb.up_out * shb.d_model
                   + shb.d_model * shb.d_ff) * wl.layers
        kvbytes = 2 * wl.batch * shb.kv_heads * (wl.pos0 + wl.seq) * shb.head_dim * 2 * wl.layers
        w8 = {"ms_per_step": round(ms8, 4), "tokens_per_s": round(wl.batch * wl.seq / (ms8 * 1e-3), 1),
              "weights": "int8 per-row symmetric, bf16 activations",
              "algorithmic_gb_per_step": round((wbytes8 + kvbytes) / 1e9, 2),
              "hbm_gbs": round((wbytes8 + kvbytes) / (ms8 * 1e-3) / 1e9, 1)}
        del layers8, descs8, model8, ws8
        torch.cuda.synchronize()

    # ---- roofline of the dominant kernel: HIP events on the launch stream around every launch
    # of each plain GEMM of one step (same shapes, same weights), repeated; the group with the
    # largest total time is reported.
    dt = torch.bfloat16 if wl.bf16 else torch.float32
    sh = wl.block
    groups = {}
    reps = 3 if args.traffic_probe else max(3, min(args.steps, 10))
    for name, M, N, K, act, count in gemm_launches(wl):
        if name == "lm_head":
            w, b = m["mw"]["wte"], None
        else:
            key = {"out": ("w_o", "b_o"), "mlp_up": ("w_up", "b_up"), "mlp_down": ("w_down", "b_down")}[name]
        x = torch.randn(M, K, device="cuda", dtype=torch.float32).to(dt)
        ld = m["logits_ld"] if name == "lm_head" else N
        y = torch.empty(M, ld, device="cuda", dtype=dt)
        res = torch.randn(M, N, device="cuda", dtype=torch.float32).to(dt) if name in ("out", "mlp_down") else None
        gws = F.workspace(F.forge_gemm_workspace_bytes(M, N, K, act, dt))
        # one event pair around each sweep over the layers' weights (the launches run back to back,
        # as they do inside a step); an event pair around every single launch would add the
        # dispatch latency on both sides to a 40 us kernel
        times = []
        for r in range(reps + 1):                 # the first sweep is a warm-up and is dropped
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for l in range(count):
                if name != "lm_head":
                    w, b = m["layers"][l][key[0]], m["layers"][l][key[1]]
                F.forge_gemm_bias_gelu(x, w, b, res, y, act, gws, n=N)
            e1.record()
            times.append((e0, e1))
        torch.cuda.synchronize()
        durs = [a.elapsed_time(b_) * 1e-3 for a, b_ in times[1:]]
        n_launch = reps * count
        nw = 2 * N if act == "swiglu" else N
        sym = "%s act=%s" % (F.forge_gemm_variant(M, N, K, act, dt, ldy=ld), act)
        gkey = sym
        gr = groups.setdefault(gkey, {"time": 0.0, "flops": 0.0, "launches": 0, "bytes": 0.0})
        gr["time"] += sum(durs)
        gr["flops"] += 2.0 * M * nw * K * n_launch
        gr["launches"] += n_launch
        del x, y, res
    if args.traffic_probe:
        return
    # ---- the fused attention call of one layer, at the workload's shape, timed the same way -------
    attn = None
    if wl.bf16:
        kvl = wl.pos0 + wl.seq
        q = torch.randn(wl.batch, sh.q_heads, wl.seq, sh.head_dim, device="cuda", dtype=torch.float32).to(dt)
        kc0, vc0 = m["kc"][0], m["vc"][0]
        o = torch.empty(wl.batch, wl.seq, sh.q_heads * sh.head_dim, device="cuda", dtype=dt)
        aws = F.workspace(F.forge_attn_fused_workspace_bytes(wl.batch, sh.q_heads, sh.kv_heads, wl.seq, kvl,
                                                             sh.head_dim, dt))
        evs = []
        per = 4                                   # calls per event pair, back to back
        for _ in range(1 + reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(per):
                F.forge_attn_fused(q, kc0, vc0, o, kv_len=kvl, workspace=aws)
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        ad = [a.elapsed_time(b) * 1e-3 / per for a, b in evs[1:]]
        at = sum(ad) / len(ad)
        if wl.seq == 1:
            kvb = 2.0 * wl.batch * sh.kv_heads * kvl * sh.head_dim * 2
            label = "attn_decode (split-KV) + combine" if aws is not None else "attn_decode (one block per kv head and sequence)"
            attn = {"kernel": label, "avg_us": round(at * 1e6, 2),
                    "hbm_gbs": round(kvb / at / 1e9, 1), "frac_of_hbm_peak": round(kvb / at / 1e9 / PEAK_HBM_GBS, 4)}
        else:
            attn = {"kernel": "attn_prefill<%d>" % sh.head_dim, "avg_us": round(at * 1e6, 2),
                    "tflops": round(attn_fl / wl.layers / at / 1e12, 1),
                    "frac_of_bf16_peak": round(attn_fl / wl.layers / at / 1e12 / PEAK_BF16_TFLOPS, 4)}
        del q, o
    dom_name, dom = max(groups.items(), key=lambda kv: kv[1]["time"])
    avg_dur = dom["time"] / dom["launches"]
    flops_per_launch = dom["flops"] / dom["launches"]
    if args.workload == "c5":
        # decode: every kernel streams weights / cache; report bytes per step over step time
        achieved = step_bytes(wl) / (ms_per_step * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None,
                    "kernel": "whole decode step (weights + KV cache read once)"}
    else:
        achieved = flops_per_launch / avg_dur / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS if wl.bf16 else 157.3,
                    "unit": "TFLOP/s", "frac": round(achieved / (PEAK_BF16_TFLOPS if wl.bf16 else 157.3), 4),
                    "traffic": recorded_traffic(wl.name, dom_name), "kernel": dom_name,
                    "avg_launch_us": round(avg_dur * 1e6, 2),
                    "launches_timed": dom["launches"],
                    "groups": {k: {"tflops": round(v["flops"] / v["time"] / 1e12, 1),
                                   "avg_us": round(v["time"] / v["launches"] * 1e6, 2)} for k, v in groups.items()}}

    # ---- the fp64 oracle on the host cores, on a bounded sample of the same workload -------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, m, args.cpu_seconds)

    line = {
        "metric": "decoder-block tokens/s; fused attention+GEMM TFLOP/s as % of MI355X peak",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if wl.bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.layers, "batch": wl.batch, "seq_len": wl.seq,
                   "kv_pos0": wl.pos0, "d_model": sh.d_model, "parallelism": "single-gpu"},
        "step_tflops": round((gemm_fl + attn_fl) / (ms_per_step * 1e-3) / 1e12, 1),
        "step_frac_of_bf16_peak": round((gemm_fl + attn_fl) / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "latency_ms": latency,
        "compiled": compiled,
        "int8_weights": w8,
        "attention": attn,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


def cpu_baseline(wl, m, budget_s):
    """Time the oracle as it stands on whole sequences of the workload until ~budget_s is spent."""
    import numpy as np
    from oracle import forge_oracle as O
    from paper_2604_16498_amd import inputs as I
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    sh = wl.block
    if sh.d_model >= 4096:
        # 8B-shaped: one layer of one sequence, scaled by the layer count
        w = {k: (None if v is None else v.float().cpu().numpy()) for k, v in m["layers"][0].items()}
        x = I.hidden_states(wl, batch=1)
        t0 = time.perf_counter()
        if wl.pos0:
            kc = m["kc"][0, :1].float().cpu().numpy().astype(np.float64)
            vc = m["vc"][0, :1].float().cpu().numpy().astype(np.float64)
            t0 = time.perf_counter()
            O.decoder_block(sh, w, x, kc, vc, pos0=wl.pos0)
        else:
            O.decoder_block(sh, w, x)
        dt_ = (time.perf_counter() - t0) * wl.layers
        return {"value": round(wl.seq / dt_, 3), "unit": "tokens/s", "cores": cores, "kind": "oracle",
                "sample": "1 layer x 1 sequence timed, multiplied by %d layers (extrapolated)" % wl.layers}
    layers = [I.block_weights(sh, wl.cid, l, wl.bf16, wl.bias_std) for l in range(wl.layers)]
    mw = I.model_weights(wl)
    done, t_used = 0, 0.0
    while done < wl.batch and t_used < budget_s:
        t0 = time.perf_counter()
        if wl.vocab:
            O.gpt_forward(sh, layers, mw, ids=m["ids_host"][done:done + 1])
        else:
            O.gpt_forward(sh, layers, mw, x=I.hidden_states(wl)[done:done + 1])
        t_used += time.perf_counter() - t0
        done += 1
    return {"value": round(done * wl.seq / t_used, 2), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%d of %d sequences of %d tokens, all %d layers%s, %.1f s" % (
                done, wl.batch, wl.seq, wl.layers, " + LM head" if wl.vocab else "", t_used)}


if __name__ == "__main__":
    main()
